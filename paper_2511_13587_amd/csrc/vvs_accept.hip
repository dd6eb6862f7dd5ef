// Acceptance stage: CFG logit mix, softmax, strict / relaxed accept test with residual resampling,
// path walk (Section 2, "Speculative Decoding"; tree verification as in Section 3).
//
// Every node of the draft tree is evaluated speculatively and in parallel - one workgroup per
// (prompt, node) computes "which child of this node is accepted, or which token is drawn if none
// is" - and a one-thread-per-prompt walk then follows the accepted children from the root.  The
// uniforms are indexed by node, so this equals the sequential procedure.
#include "vvs_device.h"

#include <limits.h>

// Phase marks: a profiling build may define VVS_PHASE_MARK(i) to record a time stamp; normally nothing.
#ifndef VVS_PHASE_MARK
#define VVS_PHASE_MARK(i)
#endif

namespace vvs {

struct AcceptArgs {
  const float* logits;        // [R][T][veff]
  const int32_t* draft;       // [B][N]
  const float* q;             // [B][T][veff]
  const float* u;             // uniforms; element (b, j, which) at b*usb + j*usj + {uoa | uot}
  int usb, usj, uoa, uot;
  const int32_t* nbr;         // [vocab][relax_k] or nullptr
  const int32_t* n_emitted;   // [B] or nullptr (no cap, never finished)
  float* probs;               // [B][T][veff] out: target distributions
  float* work;                // [B][T][2][veff] scratch: running target P and draft Q
  int32_t* node_result;       // [B][VVS_MAX_T][2] out: (accepted child or 0, drawn token or -1)
  int T, veff, lo, mode, relax_k, G;
  float scale, delta;
};

// Largest 2 * veff * 4 bytes that is kept in LDS (160 KiB per CU, a few hundred bytes are static).
constexpr size_t kAcceptLdsMax = 144 * 1024;

// Inverse CDF in ascending id: first id whose running sum exceeds u * total; if rounding runs past
// the end, the last id with mass.  Each thread owns a contiguous chunk.
__device__ int inverse_cdf(const float* __restrict__ P, int n, float u, float* red, int* ired, float* scan) {
  const int nt = blockDim.x, tid = threadIdx.x;
  const int per = (n + nt - 1) / nt;
  const int beg = min(tid * per, n), end = min(beg + per, n);
  // chunks of up to 16 ids are read once into registers (16-byte reads when the chunk is aligned)
  constexpr int CK = 16;
  float c[CK];
  const bool in_regs = per <= CK;
  float local = 0.f;
  if (in_regs) {
    if ((per & 3) == 0 && (n & 3) == 0) {
#pragma unroll
      for (int i = 0; i < CK; i += 4) {
        float4 v4 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < per && beg + i < end) v4 = *(const float4*)(P + beg + i);
        c[i] = v4.x; c[i + 1] = v4.y; c[i + 2] = v4.z; c[i + 3] = v4.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < CK; ++i) c[i] = (beg + i < end) ? P[beg + i] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < CK; ++i) local += c[i];               // ids past the chunk hold 0
  } else {
    for (int v = beg; v < end; ++v) local += P[v];
  }
  // exclusive scan of the per-thread sums: inclusive inside a wave, then wave offsets in order
  float inc = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    float t = __shfl_up(inc, o, 64);
    if ((tid & 63) >= o) inc += t;
  }
  const int w = tid >> 6, nw = nt >> 6;
  __syncthreads();
  if ((tid & 63) == 63) scan[w] = inc;
  __syncthreads();
  float woff = 0.f, total = 0.f;
  for (int i = 0; i < nw; ++i) {
    if (i < w) woff += scan[i];
    total += scan[i];
  }
  const float target = u * total;
  float run = woff + inc - local;
  int cand = INT_MAX, last_pos = -1;
  if (in_regs) {
#pragma unroll
    for (int i = 0; i < CK; ++i) {
      const float pv = c[i];
      run += pv;
      if (beg + i < end) {
        if (pv > 0.f) last_pos = beg + i;
        if (cand == INT_MAX && run > target) cand = beg + i;
      }
    }
  } else {
    for (int v = beg; v < end; ++v) {
      const float pv = P[v];
      run += pv;
      if (pv > 0.f) last_pos = v;
      if (cand == INT_MAX && run > target) cand = v;
    }
  }
  int win = block_min_int(cand, ired);
  if (win == INT_MAX) win = block_max_int(last_pos, ired);
  (void)red;
  return win;
}

// LDS_PQ: the running target and draft distributions of the node live in (dynamic) LDS, 2 * veff
// floats; otherwise in the global scratch rows.
template <bool LDS_PQ>
__global__ __launch_bounds__(1024) void k_accept_node(AcceptArgs a, TreeDesc tree) {
  extern __shared__ float pq_lds[];
  __shared__ float red[32];
  __shared__ int ired[16];
  __shared__ float scan[16];
  __shared__ float nb_mass[64];
  __shared__ int nb_id[64];
  __shared__ float sh_num, sh_px, sh_qx;
  __shared__ int sh_m;
  __shared__ int sh_cx[VVS_MAX_T];         // drafted ids (inside the slice) and accept uniforms of this node's children, in order
  __shared__ float sh_cu[VVS_MAX_T];
  __shared__ int sh_cn[VVS_MAX_T], sh_nc;  // their node ids; how many
  VVS_PHASE_MARK(0);
  const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, nt = blockDim.x;
  const int T = a.T, V = a.veff;
  const float* lc = a.logits + ((size_t)(2 * b) * T + j) * V;
  const float* lu = a.logits + ((size_t)(2 * b + 1) * T + j) * V;
  float* P = LDS_PQ ? pq_lds : a.work + ((size_t)(b * T + j) * 2) * V;
  float* Q = P + V;
  float* prow = a.probs + (size_t)(b * T + j) * V;

  // CFG mix + softmax (temperature 1) over the allowed slice.  Up to RK ids per thread (the usual
  // codebook sizes): thread tid owns ids tid + k * nt and keeps its part of the running target (and
  // later of the draft distribution) in registers for the whole kernel; the LDS / global copy P is
  // only brought up to date where ids are addressed at random (relaxed neighbourhoods, the final
  // inverse-CDF draw).  Larger slices take the generic loops over P and Q.
  constexpr int RK = 16;
  const bool regs = V <= RK * nt;
  float p[RK], q[RK];
#pragma unroll
  for (int k = 0; k < RK; ++k) p[k] = q[k] = 0.f;
  if (regs) {
    float lcv[RK], luv[RK];
#pragma unroll
    for (int k = 0; k < RK; ++k) {
      const int v = min(tid + k * nt, V - 1);                // clamped: repeats are masked below
      lcv[k] = lc[v];
      luv[k] = lu[v];
    }
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < RK; ++k) {
      p[k] = tid + k * nt < V ? luv[k] + a.scale * (lcv[k] - luv[k]) : -INFINITY;
      mx = fmaxf(mx, p[k]);
    }
    mx = block_max(mx, red);
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < RK; ++k) {
      p[k] = tid + k * nt < V ? expf(p[k] - mx) : 0.f;
      sum += p[k];
    }
    sum = block_sum(sum, red);
    const float inv_sum = 1.0f / sum;
#pragma unroll
    for (int k = 0; k < RK; ++k) {
      const int v = tid + k * nt;
      p[k] = p[k] * inv_sum;
      if (v < V) {
        P[v] = p[k];
        prow[v] = p[k];
      }
    }
  } else {
    float mx = -INFINITY;
    for (int v = tid; v < V; v += nt) {
      const float m = lu[v] + a.scale * (lc[v] - lu[v]);
      P[v] = m;
      mx = fmaxf(mx, m);
    }
    mx = block_max(mx, red);
    float sum = 0.f;
    for (int v = tid; v < V; v += nt) {
      const float e = expf(P[v] - mx);
      P[v] = e;
      sum += e;
    }
    sum = block_sum(sum, red);
    for (int v = tid; v < V; v += nt) {
      const float pv = P[v] / sum;
      P[v] = pv;
      prow[v] = pv;
    }
  }
  __syncthreads();

  VVS_PHASE_MARK(1);
  int32_t* res = a.node_result + ((size_t)b * VVS_MAX_T + j) * 2;
  int cap = INT_MAX;
  if (a.n_emitted) {
    const int ne = a.n_emitted[b];
    if (ne >= a.G) {                       // image complete: nothing to accept, nothing to draw
      if (tid == 0) { res[0] = 0; res[1] = -1; }
      return;
    }
    cap = a.G - ne - 1;
  }

  int accepted = 0;
  bool p_in_memory = true;                   // P holds the current target (false: only the registers do)
  if (tree.first_child[j] >= 0 && tree.depth[j] < cap && tree.first_child[j] <= tree.n_forced) {
    accepted = tree.first_child[j];          // post verification: accepted without a test, nothing is read or changed
  } else if (tree.first_child[j] >= 0 && tree.depth[j] < cap) {
    const float* qrow = a.q + (size_t)(b * T + j) * V;
    const int N = T - 1;
    // the children (ascending node id = the order in which they are tried), their drafted ids and
    // uniforms: found by the first wave in parallel, one memory round trip for all of them
    if (tid < VVS_MAX_T) {
      const bool child = tid > 0 && tid < T && tree.parent[tid] == j;
      const unsigned long long m = __ballot(child);
      if (child) {
        const int rank = __popcll(m & ((1ull << tid) - 1ull));
        sh_cn[rank] = tid;
        sh_cx[rank] = min(max(a.draft[b * N + tid - 1] - a.lo, 0), V - 1);
        sh_cu[rank] = a.u[(size_t)b * a.usb + (size_t)tid * a.usj + a.uoa];
      }
      if (tid == 0) sh_nc = __popcll(m);
    }
    if (regs) {
#pragma unroll
      for (int k = 0; k < RK; ++k) q[k] = tid + k * nt < V ? qrow[tid + k * nt] : 0.f;
    } else {
      for (int v0 = tid; v0 < V; v0 += 8 * nt) {             // 8 independent requests per thread and pass
        float qv[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) qv[k] = qrow[min(v0 + k * nt, V - 1)];
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (v0 + k * nt < V) Q[v0 + k * nt] = qv[k];
      }
    }
    __syncthreads();
    const int n_children = sh_nc;
    for (int ci = 0; ci < n_children; ++ci) {
      const int c = sh_cn[ci];
      const int x = sh_cx[ci];
      const float ua = sh_cu[ci];
      const int xo = x % nt, xk = x / nt;                    // owner thread and register of id x
      if (a.mode == VVS_RELAXED && a.relax_k > 0) {
        // absorb neighbour mass in ascending distance while the absorbed total stays <= delta
        if (regs && !p_in_memory) {
#pragma unroll
          for (int k = 0; k < RK; ++k)
            if (tid + k * nt < V) P[tid + k * nt] = p[k];
          __syncthreads();
          p_in_memory = true;
        }
        if (tid < 64) {
          float pm = 0.f;
          int id = -1;
          if (tid < a.relax_k) {
            id = a.nbr[(size_t)(a.lo + x) * a.relax_k + tid] - a.lo;
            if (id >= 0 && id < V) pm = P[id]; else id = -1;
          }
          nb_mass[tid] = pm;
          nb_id[tid] = id;
        }
        __syncthreads();
        if (tid == 0) {
          float absorbed = 0.f;
          int m = 0;
          for (; m < a.relax_k; ++m) {
            if (nb_id[m] < 0) continue;
            if (absorbed + nb_mass[m] > a.delta) break;
            absorbed += nb_mass[m];
          }
          sh_m = m;
          sh_num = P[x] + absorbed;
        }
        __syncthreads();
        if (tid < sh_m && nb_id[tid] >= 0) P[nb_id[tid]] = 0.f;
        __syncthreads();
        if (tid == 0) P[x] = sh_num;
        __syncthreads();
        if (regs) {
#pragma unroll
          for (int k = 0; k < RK; ++k)
            if (tid + k * nt < V) p[k] = P[tid + k * nt];
        }
      }
      float num, qx;
      if (regs) {                                            // the owner of id x publishes its target and draft mass
        if (tid == xo) {
          float pv = 0.f, qv = 0.f;
#pragma unroll
          for (int k = 0; k < RK; ++k)
            if (k == xk) { pv = p[k]; qv = q[k]; }
          sh_px = pv;
          sh_qx = qv;
        }
        __syncthreads();
        num = sh_px;
        qx = sh_qx;
      } else {
        num = P[x];
        qx = Q[x];
      }
      if (ua * qx < num) { accepted = c; break; }
      // rejected: target <- normalised positive part of (target - draft); drop x from the draft
      if (regs) {
        float r[RK];
        float z = 0.f, zq = 0.f;
#pragma unroll
        for (int k = 0; k < RK; ++k) {
          r[k] = fmaxf(0.f, p[k] - q[k]);
          if (tid == xo && k == xk) q[k] = 0.f;              // x leaves the draft distribution
          z += r[k];
          zq += q[k];
        }
        const float2 zz = block_sum2(z, zq, red);
        if (zz.x > 0.f) {                                    // a residual without mass leaves the target as it is
          const float inv = 1.0f / zz.x;                       // one division per row instead of one per id: 16 waves share 4 SIMDs
#pragma unroll
          for (int k = 0; k < RK; ++k) p[k] = r[k] * inv;
          p_in_memory = false;
        }
        if (!(zz.y > 0.f)) break;
        const float invq = 1.0f / zz.y;
#pragma unroll
        for (int k = 0; k < RK; ++k) q[k] = q[k] * invq;
      } else {
        float z = 0.f;
        for (int v = tid; v < V; v += nt) z += fmaxf(0.f, P[v] - Q[v]);
        z = block_sum(z, red);
        if (z > 0.f)
          for (int v = tid; v < V; v += nt) P[v] = fmaxf(0.f, P[v] - Q[v]) / z;
        __syncthreads();
        if (tid == 0) Q[x] = 0.f;
        __syncthreads();
        float zq = 0.f;
        for (int v = tid; v < V; v += nt) zq += Q[v];
        zq = block_sum(zq, red);
        if (!(zq > 0.f)) break;
        for (int v = tid; v < V; v += nt) Q[v] = Q[v] / zq;
        __syncthreads();
      }
    }
  }
  VVS_PHASE_MARK(2);
  if (accepted) {
    if (tid == 0) { res[0] = accepted; res[1] = -1; }
    return;
  }
  if (regs && !p_in_memory) {                                // the draw addresses ids in ascending order: bring P up to date
    __syncthreads();
#pragma unroll
    for (int k = 0; k < RK; ++k)
      if (tid + k * nt < V) P[tid + k * nt] = p[k];
  }
  __syncthreads();
  const float ut = a.u[(size_t)b * a.usb + (size_t)j * a.usj + a.uot];
  const int tok = inverse_cdf(P, V, ut, red, ired, scan);
  VVS_PHASE_MARK(3);
  if (tid == 0) { res[0] = 0; res[1] = a.lo + tok; }
}

// Follows accepted children from the root: one wave per prompt, lane 0 walks (at most tree-depth
// dependent reads), then the lanes write one path entry each.
__global__ __launch_bounds__(64) void k_walk(const int32_t* __restrict__ node_result, int B, int32_t* __restrict__ accept_len,
                                             int32_t* __restrict__ path, int32_t* __restrict__ next_token, int32_t* __restrict__ keep) {
  static_assert(VVS_MAX_T == 64, "one lane per path entry");
  __shared__ int p[VVS_MAX_T];
  __shared__ int s_a, s_tok;
  const int b = blockIdx.x, i = threadIdx.x;
  if (i == 0) {
    int cur = 0, a = 0;
    p[0] = 0;
    while (a < VVS_MAX_T - 1) {
      const int nxt = node_result[((size_t)b * VVS_MAX_T + cur) * 2];
      if (nxt <= cur) break;               // 0 = nothing accepted (children always have larger ids)
      cur = nxt;
      p[++a] = cur;
    }
    s_a = a;
    s_tok = node_result[((size_t)b * VVS_MAX_T + cur) * 2 + 1];
  }
  __syncthreads();
  const int a = s_a, tok = s_tok;
  if (i == 0) {
    if (accept_len) accept_len[b] = a;
    if (next_token) next_token[b] = tok;
    if (keep) { keep[b] = a; keep[B + b] = tok; }
  }
  const int v = i <= a ? p[i] : -1;
  if (path) path[b * VVS_MAX_T + i] = v;
  if (keep) keep[2 * B + b * VVS_MAX_T + i] = v;
}

static void launch_accept_on(Ctx* c, const TreeDesc& tree, int T, const float* d_logits, const int32_t* d_draft_tokens, const float* d_q,
                             const float* d_u, int usb, int usj, int uoa, int uot, int mode, bool use_state, int32_t* d_accept_len,
                             int32_t* d_path, int32_t* d_next, int32_t* keep, float* probs, float* work, int32_t* node_result, hipStream_t s) {
  Timed timed(c, VVS_K_ACCEPT, s);
  AcceptArgs a;
  a.logits = d_logits; a.draft = d_draft_tokens; a.q = d_q; a.u = d_u;
  a.usb = usb; a.usj = usj; a.uoa = uoa; a.uot = uot;
  a.nbr = c->nbr;
  a.n_emitted = use_state ? (const int32_t*)(c->ws + c->w.state) + c->B : nullptr;
  a.probs = probs;
  a.work = work;
  a.node_result = node_result;
  a.T = T; a.veff = c->veff; a.lo = c->lo; a.mode = mode; a.relax_k = c->cfg.relax_k; a.G = c->G;
  a.scale = c->cfg.cfg_scale; a.delta = c->cfg.relax_delta;
  const size_t pq_bytes = (size_t)2 * c->veff * sizeof(float);
  if (pq_bytes <= kAcceptLdsMax) {
    if (pq_bytes > 64 * 1024) allow_dynamic_lds((const void*)k_accept_node<true>, kAcceptLdsMax);
    hipLaunchKernelGGL(k_accept_node<true>, dim3(T, c->B), dim3(1024), pq_bytes, s, a, tree);
  } else {
    hipLaunchKernelGGL(k_accept_node<false>, dim3(T, c->B), dim3(1024), 0, s, a, tree);
  }
  hipLaunchKernelGGL(k_walk, dim3(c->B), dim3(64), 0, s, (const int32_t*)a.node_result, c->B, d_accept_len, d_path, d_next, keep);
}

void launch_accept(Ctx* c, const TreeDesc& tree, int T, const float* d_logits, const int32_t* d_draft_tokens, const float* d_q,
                   const float* d_u, int usb, int usj, int uoa, int uot, int mode, bool use_state, int32_t* d_accept_len,
                   int32_t* d_path, int32_t* d_next, bool keep_outcome, hipStream_t s) {
  launch_accept_on(c, tree, T, d_logits, d_draft_tokens, d_q, d_u, usb, usj, uoa, uot, mode, use_state, d_accept_len, d_path, d_next,
                   keep_outcome ? (int32_t*)(c->ws + c->w.outcome) : nullptr, (float*)(c->ws + c->w.probs), (float*)(c->ws + c->w.pq_work),
                   (int32_t*)(c->ws + c->w.node_result), s);
}

// ------------------------------------------------------------------------------------------------ acceptance stage without any allocation
// The acceptance stage for callers that cannot allocate device memory and have no workspace to hand over: its
// two scratch buffers - the per-node results between k_accept_node and k_walk, and the per-node target
// distributions k_accept_node writes - live in one static device array.  Every GPU holds its own copy of the
// array at its own address; the address is looked up once per device (hipGetSymbolAddress, with that device
// current) and kept.  Nothing in the array has to start at zero: k_accept_node writes every entry that k_walk
// or a later phase reads.  Two calls that overlap on one GPU (two streams, two contexts) share the array and race.
constexpr size_t kNoAllocNodeBytes = (size_t)VVS_NOALLOC_MAX_PROMPTS * VVS_MAX_T * 2 * sizeof(int32_t);
constexpr size_t kNoAllocProbBytes = (size_t)VVS_NOALLOC_MAX_PROB_FLOATS * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kNoAllocNodeBytes + kNoAllocProbBytes];

constexpr int kMaxDevices = 64;
static unsigned char* g_scratch_ptr[kMaxDevices];   // per device: address of that device's copy of `scratch`

vvs_status launch_accept_noalloc(Ctx* c, const TreeDesc& tree, int T, const float* d_logits, const int32_t* d_draft_tokens,
                                 const float* d_q, const float* d_u, int mode, int32_t* d_accept_len, int32_t* d_path, int32_t* d_next,
                                 hipStream_t s, std::string* err) {
  if (c->B > VVS_NOALLOC_MAX_PROMPTS || (size_t)c->B * T * c->veff > (size_t)VVS_NOALLOC_MAX_PROB_FLOATS) {
    *err = "accept_from_logits_noalloc: n_prompts * (n_nodes + 1) * V_eff exceeds VVS_NOALLOC_MAX_PROB_FLOATS (or n_prompts exceeds "
           "VVS_NOALLOC_MAX_PROMPTS): the static scratch array is too small for this call";
    return VVS_ESIZE;
  }
  if ((size_t)2 * c->veff * sizeof(float) > kAcceptLdsMax) {
    *err = "accept_from_logits_noalloc: the allowed-id slice is too wide for the LDS-resident acceptance kernel";
    return VVS_ESIZE;
  }
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) { *err = "accept_from_logits_noalloc: hipGetDevice failed"; return VVS_EHIP; }
  if (!g_scratch_ptr[dev]) {
    unsigned char* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      *err = std::string("accept_from_logits_noalloc: hipGetSymbolAddress: ") + hipGetErrorString(e);
      return VVS_EHIP;
    }
    g_scratch_ptr[dev] = p;
  }
  unsigned char* base = g_scratch_ptr[dev];
  launch_accept_on(c, tree, T, d_logits, d_draft_tokens, d_q, d_u, 2 * T, 2, 0, 1, mode, false, d_accept_len, d_path, d_next, nullptr,
                   (float*)(base + kNoAllocNodeBytes), nullptr, (int32_t*)base, s);
  return VVS_OK;
}

__global__ void k_prefill_finish(const int32_t* __restrict__ node_result, int32_t* __restrict__ state, int32_t* __restrict__ first,
                                 int B, int kv_len, int n_emitted) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int tok = node_result[((size_t)b * VVS_MAX_T) * 2 + 1];
  first[b] = tok;
  state[b] = kv_len;
  state[B + b] = n_emitted;
  state[2 * B + b] = tok;
}

void launch_prefill_finish(Ctx* c, int n_forced, int32_t* d_first, hipStream_t s) {
  hipLaunchKernelGGL(k_prefill_finish, dim3((c->B + 63) / 64), dim3(64), 0, s, (const int32_t*)(c->ws + c->w.node_result),
                     (int32_t*)(c->ws + c->w.state), d_first, c->B, c->P + n_forced, n_forced + 1);
}

}  // namespace vvs
