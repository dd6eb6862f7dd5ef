// Weighted average similarity of the candidate paths of a draft tree (Section 4.4, Eq. 2; Algorithm 1:
// "Downsample" with stride 2, then "CompSim") - the quantity the dynamic schedule compares with its
// threshold to decide whether a step may skip verification.
//
// One wave per prompt.  The tree comes by value; the kept paths (every stride-th leaf in leaf order)
// are laid out in LDS as node ids per position, then for every position the cosine similarities of
// the codebook embeddings of all unordered pairs of paths that reach it are averaged, and the
// positions are combined with weights proportional to alpha^position.  The data is a few hundred
// bytes per prompt: the kernel is latency-bound by construction (two dependent reads: token id, then
// its embedding); sums are kept in double so that the result does not depend on the pair order.
#include "vvs_device.h"

namespace vvs {

__global__ __launch_bounds__(64) void k_path_similarity(TreeDesc tree, int n_nodes, const int32_t* __restrict__ tokens,
                                                        const float* __restrict__ embed, int dim, float alpha, int stride,
                                                        float* __restrict__ out) {
  __shared__ int8_t s_node[VVS_MAX_T][VVS_MAX_T];     // [path][position] -> node id
  __shared__ int s_len[VVS_MAX_T];
  __shared__ int s_leaf[VVS_MAX_T];
  __shared__ int s_np;
  const int b = blockIdx.x, lane = threadIdx.x;
  if (lane == 0) {                                     // kept leaves: every stride-th one in ascending node id
    int seen = 0, np = 0;
    for (int j = 1; j <= n_nodes; ++j)
      if (tree.first_child[j] < 0) {
        if (seen % stride == 0) s_leaf[np++] = j;
        ++seen;
      }
    s_np = np;
  }
  __syncthreads();
  const int np = s_np;
  int lmax = 0;
  for (int p = lane; p < np; p += 64) {                // one path per lane: walk up from the leaf
    int node = s_leaf[p];
    const int len = tree.depth[node];
    s_len[p] = len;
    for (int k = len - 1; k >= 0; --k) {
      s_node[p][k] = (int8_t)node;
      node = tree.parent[node];
    }
  }
  __syncthreads();
  for (int p = 0; p < np; ++p) lmax = max(lmax, s_len[p]);
  double num = 0.0, den = 0.0, wl = 1.0;
  for (int l = 0; l < lmax; ++l, wl *= (double)alpha) {
    double total = 0.0;
    int pairs = 0;
    for (int idx = lane; idx < np * np; idx += 64) {
      const int i = idx / np, j = idx % np;
      if (i >= j || s_len[i] <= l || s_len[j] <= l) continue;
      const float* ea = embed + (size_t)tokens[(size_t)b * n_nodes + s_node[i][l] - 1] * dim;
      const float* eb = embed + (size_t)tokens[(size_t)b * n_nodes + s_node[j][l] - 1] * dim;
      double ab = 0.0, aa = 0.0, bb = 0.0;
      for (int k = 0; k < dim; ++k) {
        const double x = ea[k], y = eb[k];
        ab += x * y; aa += x * x; bb += y * y;
      }
      total += (aa > 0.0 && bb > 0.0) ? ab / (sqrt(aa) * sqrt(bb)) : 0.0;
      ++pairs;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      total += __shfl_xor(total, o, 64);
      pairs += __shfl_xor(pairs, o, 64);
    }
    if (pairs > 0) {                                   // positions that fewer than two paths reach are left out
      num += wl * (total / pairs);
      den += wl;
    }
  }
  if (lane == 0) out[b] = den > 0.0 ? (float)(num / den) : 1.0f;
}

void launch_path_similarity(Ctx* c, const TreeDesc& tree, int n_nodes, const int32_t* d_draft_tokens, float alpha, int stride,
                            float* d_similarity, hipStream_t s) {
  Timed timed(c, VVS_K_ELEMENTWISE, s);
  hipLaunchKernelGGL(k_path_similarity, dim3(c->B), dim3(64), 0, s, tree, n_nodes, d_draft_tokens, c->codebook, c->code_dim, alpha,
                     stride, d_similarity);
}

}  // namespace vvs
