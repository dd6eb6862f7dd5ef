// Element-wise / reduction kernels of the verify pass, the fp32 (reference-shape) GEMM and attention
// kernels, weight repacking, KV commit, and the launch sequence of one transformer forward.
// The bf16 GEMM and attention kernels (MFMA) live in vvs_mfma.hip; the acceptance stage in
// vvs_accept.hip.
#include "vvs_device.h"

#include <stdlib.h>
#include <algorithm>

namespace vvs {

// ------------------------------------------------------------------------------------------------ utilities
__global__ void k_fill_zero(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const uint4 z = make_uint4(0, 0, 0, 0);
  for (; i < n16; i += stride) p[i] = z;
}

void launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  size_t n16 = bytes / 16;
  if (!n16) return;
  int blocks = (int)std::min<size_t>((n16 + 255) / 256, 256 * 32);
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, s, (uint4*)p, n16);
}

__global__ void k_copy_bytes(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) dst[i] = src[i];
}

void launch_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s) {
  size_t n16 = bytes / 16;
  if (!n16) return;
  int blocks = (int)std::min<size_t>((n16 + 255) / 256, 256 * 32);
  hipLaunchKernelGGL(k_copy_bytes, dim3(blocks), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n16);
}

// out[n][k] = in[k][col0 + n]   (in: [K][ld])
template <typename T>
__global__ void k_transpose(const T* __restrict__ in, T* __restrict__ out, int K, int N, int ld, int col0) {
  __shared__ T tile[32][33];
  const int n0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
  for (int i = threadIdx.y; i < 32; i += 8) {
    int k = k0 + i, n = n0 + threadIdx.x;
    if (k < K && n < N) tile[i][threadIdx.x] = in[(size_t)k * ld + col0 + n];
  }
  __syncthreads();
  for (int i = threadIdx.y; i < 32; i += 8) {
    int n = n0 + i, k = k0 + threadIdx.x;
    if (k < K && n < N) out[(size_t)n * K + k] = tile[threadIdx.x][i];
  }
}

// bf16 weights: out = packed fragment order of W^T, i.e. rows = output features n, contraction = k;
// in[k][col0 + n].  One thread per 16-byte chunk; the 32 lanes of a half-block read 32 consecutive n.
// Row block nb of the source lands in row block nb * nb_stride + nb_off of the destination (gate and
// up projections are interleaved block by block so that one GEMM tile holds both for the same units).
// The weights are copied bit for bit: the packed operand holds exactly the bf16 values the caller gave.
__global__ void k_pack_w(const bf16_t* __restrict__ in, uint4* __restrict__ out, int K, int N, int ld, int col0, int nb_stride,
                         int nb_off) {
  const size_t chunk = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)(N >> 5) * (K >> 4) * 64;
  if (chunk >= total) return;
  const int lane = (int)(chunk & 63);
  const size_t blk = chunk >> 6;
  const int kb = (int)(blk % (K >> 4)), nb = (int)(blk / (K >> 4));
  const int n = nb * 32 + (lane & 31), k0 = kb * 16 + (lane >> 5) * 8;
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = in[(size_t)(k0 + 2 * i) * ld + col0 + n], hi = in[(size_t)(k0 + 2 * i + 1) * ld + col0 + n];
    w[i] = lo | (hi << 16);
  }
  out[(((size_t)nb * nb_stride + nb_off) * (K >> 4) + kb) * 64 + lane] = make_uint4(w[0], w[1], w[2], w[3]);
}

// bf16 activations, row-major [M][K] -> packed fragment order (rows beyond M are zero)
__global__ void k_pack_a(const bf16_t* __restrict__ in, uint4* __restrict__ out, int M, int K) {
  const size_t chunk = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)((M + 31) >> 5) * (K >> 4) * 64;
  if (chunk >= total) return;
  const int lane = (int)(chunk & 63);
  const size_t blk = chunk >> 6;
  const int kb = (int)(blk % (K >> 4)), mb = (int)(blk / (K >> 4));
  const int m = mb * 32 + (lane & 31), k0 = kb * 16 + (lane >> 5) * 8;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (m < M) v = *(const uint4*)(in + (size_t)m * K + k0);
  out[chunk] = v;
}

template <typename T>
static void transpose_into(const void* in, void* out, int K, int N, int ld, int col0, hipStream_t s, int nb_stride = 1, int nb_off = 0) {
  if (sizeof(T) == 2) {
    const size_t total = (size_t)(N >> 5) * (K >> 4) * 64;
    hipLaunchKernelGGL(k_pack_w, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t*)in, (uint4*)out, K, N, ld, col0,
                       nb_stride, nb_off);
    return;
  }
  dim3 grid((N + 31) / 32, (K + 31) / 32);
  hipLaunchKernelGGL(k_transpose<T>, grid, dim3(32, 8), 0, s, (const T*)in, (T*)out, K, N, ld, col0);
}

template <typename T>
__global__ void k_copy(const T* __restrict__ in, T* __restrict__ out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i < n; i += (size_t)gridDim.x * blockDim.x) out[i] = in[i];
}
template <typename T>
__global__ void k_to_float(const T* __restrict__ in, float* __restrict__ out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i < n; i += (size_t)gridDim.x * blockDim.x) out[i] = ld(in + i);
}

template <typename T>
static void pack_weights_t(Ctx* c, const void* const* t, hipStream_t s) {
  const int d = c->d, F = c->F;
  auto copy = [&](const void* in, size_t off, size_t n) {
    int blocks = (int)std::min<size_t>((n + 255) / 256, 8192);
    hipLaunchKernelGGL(k_copy<T>, dim3(blocks), dim3(256), 0, s, (const T*)in, (T*)(c->pw + off), n);
  };
  auto gain = [&](const void* in, size_t off) {
    hipLaunchKernelGGL(k_to_float<T>, dim3((d + 255) / 256), dim3(256), 0, s, (const T*)in, (float*)(c->pw + off), (size_t)d);
  };
  copy(t[0], c->p.embed, (size_t)c->V * d);
  if (t[1]) copy(t[1], c->p.prefix_embed, (size_t)(c->cfg.n_classes + 1) * d);
  for (int l = 0; l < c->L; ++l) {
    const void* const* w = t + 2 + 9 * l;
    size_t base = c->p.layer0 + c->p.layer_stride * l;
    gain(w[0], base + c->p.g1);
    char* qkv = c->pw + base + c->p.wqkv;
    for (int i = 0; i < 3; ++i) transpose_into<T>(w[1 + i], qkv + (size_t)i * d * d * sizeof(T), d, d, d, 0, s);
    transpose_into<T>(w[4], c->pw + base + c->p.wo, d, d, d, 0, s);
    gain(w[5], base + c->p.g2);
    char* gu = c->pw + base + c->p.wgu;
    if (sizeof(T) == 2) {            // bf16: gate / up interleaved in blocks of 32 output features
      transpose_into<T>(w[6], gu, d, F, F, 0, s, 2, 0);
      transpose_into<T>(w[7], gu, d, F, F, 0, s, 2, 1);
    } else {
      transpose_into<T>(w[6], gu, d, F, F, 0, s);
      transpose_into<T>(w[7], gu + (size_t)F * d * sizeof(T), d, F, F, 0, s);
    }
    transpose_into<T>(w[8], c->pw + base + c->p.wd, F, d, d, 0, s);
  }
  const void* const* tail = t + 2 + 9 * c->L;
  gain(tail[0], c->p.gf);
  transpose_into<T>(tail[1], c->pw + c->p.wout, d, c->veff, c->V, c->lo, s);
  if (c->cfg.draft_input) transpose_into<T>(tail[2], c->pw + c->p.fc, 2 * d, d, d, 0, s);
}

void launch_pack_weights(Ctx* c, const void* const* tensors, hipStream_t s) {
  if (c->cfg.dtype == VVS_BF16) pack_weights_t<bf16_t>(c, tensors, s);
  else pack_weights_t<float>(c, tensors, s);
}

// ------------------------------------------------------------------------------------------------ embedding
struct EmbedArgs {
  int T, d, V, mode;                 // mode 0: verify (token table), 1: prefill chunk
  const int32_t* tokens_bt;          // [B][T]
  const void* pc; const void* pu;    // prefix inputs
  int prefix_kind, n_classes, P, chunk_start, n_forced;
  const int32_t* forced;
};

template <typename T>
__device__ __forceinline__ const T* embed_source(const T* __restrict__ embed, const T* __restrict__ prefix_tab, const EmbedArgs& a, int m) {
  const int r = m / a.T, t = m % a.T, b = r >> 1;
  const T* src;
  if (a.mode == 0) {
    int tok = min(max(a.tokens_bt[b * a.T + t], 0), a.V - 1);
    src = embed + (size_t)tok * a.d;
  } else {
    int slot = a.chunk_start + t;
    if (slot < a.P) {
      if (a.prefix_kind == VVS_PREFIX_CLASS) {
        int id;
        if (r & 1) id = a.pu ? ((const int32_t*)a.pu)[b * a.P + slot] : a.n_classes;
        else id = ((const int32_t*)a.pc)[b * a.P + slot];
        id = min(max(id, 0), a.n_classes);
        src = prefix_tab + (size_t)id * a.d;
      } else {
        src = (r & 1) ? (const T*)a.pu + (size_t)slot * a.d : (const T*)a.pc + ((size_t)b * a.P + slot) * a.d;
      }
    } else {
      int tok = min(max(a.forced[b * a.n_forced + slot - a.P], 0), a.V - 1);
      src = embed + (size_t)tok * a.d;
    }
  }
  return src;
}

template <typename T>
__global__ void k_embed(float* __restrict__ x, const T* __restrict__ embed, const T* __restrict__ prefix_tab, EmbedArgs a) {
  const int m = blockIdx.x;
  const T* src = embed_source(embed, prefix_tab, a, m);
  for (int i = threadIdx.x; i < a.d; i += blockDim.x) x[(size_t)m * a.d + i] = ld(src + i);
}

// Embedding for the path without separate normalisation kernels: x (fp32), bf16(x * g) in packed operand
// order (g = gain of the norm that follows), and the row's sum of squares (slab 0 holds the whole sum, the
// other slabs 0).
__global__ __launch_bounds__(256) void k_embed_packed(float* __restrict__ x, bf16_t* __restrict__ xb, float* __restrict__ ss, int NS,
                                                      const bf16_t* __restrict__ embed, const bf16_t* __restrict__ prefix_tab,
                                                      const float* __restrict__ g, EmbedArgs a, int pad_T, int pad) {
  __shared__ float red[16];
  const int m = blockIdx.x;
  const int mp = pad_T > 0 ? (m / pad_T) * pad + m % pad_T : m;   // row of the packed operand (row-padded layout: pad rows per pad_T tokens)
  const bf16_t* src = embed_source(embed, prefix_tab, a, m);
  float sq = 0.f;
  for (int k0 = threadIdx.x * 8; k0 < a.d; k0 += 256 * 8) {
    const uint4 raw = *(const uint4*)(src + k0);
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    float v[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = bf2f((bf16_t)(w[i] & 0xFFFF)); v[2 * i + 1] = bf2f((bf16_t)(w[i] >> 16)); }
    store8(x, m, k0, a.d, v);
    const float4 ga = *(const float4*)(g + k0), gb = *(const float4*)(g + k0 + 4);
    const float hv[8] = {v[0] * ga.x, v[1] * ga.y, v[2] * ga.z, v[3] * ga.w, v[4] * gb.x, v[5] * gb.y, v[6] * gb.z, v[7] * gb.w};
    store8(xb, mp, k0, a.d, hv);
#pragma unroll
    for (int i = 0; i < 8; ++i) sq += v[i] * v[i];
  }
  sq = block_sum(sq, red);
  if (threadIdx.x < NS) ss[(size_t)m * NS + threadIdx.x] = threadIdx.x == 0 ? sq : 0.f;
}

// Rows (i * stride + off) of x, times the gain g -> packed bf16 rows i, with their sums of squares (for the lm_head of a prefill)
__global__ __launch_bounds__(256) void k_gather_rows(const float* __restrict__ x, const float* __restrict__ ss, const float* __restrict__ g,
                                                     bf16_t* __restrict__ xb2, float* __restrict__ ss2, int d, int NS, int stride, int off) {
  const int i = blockIdx.x;
  const size_t m = (size_t)i * stride + off;
  for (int k0 = threadIdx.x * 8; k0 < d; k0 += 256 * 8) {
    const float4 a = *(const float4*)(x + m * d + k0), b = *(const float4*)(x + m * d + k0 + 4);
    const float4 ga = *(const float4*)(g + k0), gb = *(const float4*)(g + k0 + 4);
    const float v[8] = {a.x * ga.x, a.y * ga.y, a.z * ga.z, a.w * ga.w, b.x * gb.x, b.y * gb.y, b.z * gb.z, b.w * gb.w};
    store8(xb2, i, k0, d, v);
  }
  if (threadIdx.x < NS) ss2[(size_t)i * NS + threadIdx.x] = ss[m * NS + threadIdx.x];
}

__global__ void k_build_tokens(int32_t* __restrict__ tokens, const int32_t* __restrict__ pending, const int32_t* __restrict__ draft,
                               int B, int T) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * T) return;
  int b = i / T, j = i % T;
  tokens[i] = j == 0 ? pending[b] : draft[b * (T - 1) + j - 1];
}

void launch_build_tokens(Ctx* c, int T, const int32_t* d_draft, hipStream_t s) {
  Timed timed(c, VVS_K_ELEMENTWISE, s);
  int n = c->B * T;
  const int32_t* pending = (const int32_t*)(c->ws + c->w.state) + 2 * c->B;
  hipLaunchKernelGGL(k_build_tokens, dim3((n + 255) / 256), dim3(256), 0, s, (int32_t*)(c->ws + c->w.tokens), pending, d_draft,
                     c->B, T);
}

// ------------------------------------------------------------------------------------------------ residual add + RMSNorm
// Output row i reads x row (i * in_stride + in_off): x_row += sum of GEMM partials (if any), then
// h_row = x_row / sqrt(mean(x_row^2) + eps) * g, rounded to the operand type.
template <typename T, int NCH, int NT>
__global__ __launch_bounds__(NT) void k_add_rmsnorm(float* __restrict__ x, const float* __restrict__ partial, int splits,
                                                     size_t split_stride, int d, const float* __restrict__ g, float eps,
                                                     T* __restrict__ h, int in_stride, int in_off) {
  // each of the NT threads owns NCH chunks of 8 consecutive values of the row (d <= NCH * NT * 8) and keeps them in
  // registers between the sum of squares and the scaling; one chunk per thread where the row allows it, so that
  // everything a row needs is requested in one round trip to memory
  __shared__ float red[16];
  const size_t row = (size_t)blockIdx.x * in_stride + in_off;
  float* xr = x + row * d;
  float xv[NCH][8];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int k0 = (threadIdx.x + NT * j) * 8;
    if (k0 < d) {
      const float4 a = *(const float4*)(xr + k0), b = *(const float4*)(xr + k0 + 4);
      float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
      if (splits) {
        // all partial sums of the chunk are requested before the first is added (the planner makes at most 8 splits): one
        // round trip to memory per chunk instead of one per split; added in the order of the splits
        constexpr int kMaxSplits = 8;
        float4 pa[kMaxSplits], pb[kMaxSplits];
#pragma unroll
        for (int s = 0; s < kMaxSplits; ++s) {
          if (s < splits) {
            const float* pr = partial + s * split_stride + row * d + k0;
            pa[s] = *(const float4*)pr;
            pb[s] = *(const float4*)(pr + 4);
          }
        }
#pragma unroll
        for (int s = 0; s < kMaxSplits; ++s) {
          if (s < splits) {
            v[0] += pa[s].x; v[1] += pa[s].y; v[2] += pa[s].z; v[3] += pa[s].w;
            v[4] += pb[s].x; v[5] += pb[s].y; v[6] += pb[s].z; v[7] += pb[s].w;
          }
        }
        for (int s = kMaxSplits; s < splits; ++s) {          // not reached with the planner's limit
          const float* pr = partial + s * split_stride + row * d + k0;
          const float4 qa = *(const float4*)pr, qb = *(const float4*)(pr + 4);
          v[0] += qa.x; v[1] += qa.y; v[2] += qa.z; v[3] += qa.w; v[4] += qb.x; v[5] += qb.y; v[6] += qb.z; v[7] += qb.w;
        }
        *(float4*)(xr + k0) = make_float4(v[0], v[1], v[2], v[3]);
        *(float4*)(xr + k0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) { xv[j][i] = v[i]; ss += v[i] * v[i]; }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) xv[j][i] = 0.f;
    }
  }
  ss = block_sum(ss, red);
  const float scale = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int k0 = (threadIdx.x + NT * j) * 8;
    if (k0 < d) {
      float gv[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
      if (g) {
        const float4 ga = *(const float4*)(g + k0), gb = *(const float4*)(g + k0 + 4);
        gv[0] = ga.x; gv[1] = ga.y; gv[2] = ga.z; gv[3] = ga.w; gv[4] = gb.x; gv[5] = gb.y; gv[6] = gb.z; gv[7] = gb.w;
      }
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = xv[j][i] * scale * gv[i];
      store8(h, (int)blockIdx.x, k0, d, v);
    }
  }
}

template <typename T>
static void launch_add_rmsnorm(int rows, float* x, const float* partial, int splits, size_t split_stride, int d, const float* g, float eps,
                               T* h, int in_stride, int in_off, hipStream_t s) {
  if (d <= 2048)
    hipLaunchKernelGGL((k_add_rmsnorm<T, 1, 256>), dim3(rows), dim3(256), 0, s, x, partial, splits, split_stride, d, g, eps, h, in_stride, in_off);
  else if (d <= 4096)
    hipLaunchKernelGGL((k_add_rmsnorm<T, 1, 512>), dim3(rows), dim3(512), 0, s, x, partial, splits, split_stride, d, g, eps, h, in_stride, in_off);
  else
    hipLaunchKernelGGL((k_add_rmsnorm<T, 8, 256>), dim3(rows), dim3(256), 0, s, x, partial, splits, split_stride, d, g, eps, h, in_stride, in_off);
}

// ------------------------------------------------------------------------------------------------ RoPE + KV write
template <typename T>
__global__ void k_rope_kv(const float* __restrict__ qkv, int splits, size_t split_stride, T* __restrict__ q, T* __restrict__ kc,
                          T* __restrict__ vc, const float* __restrict__ rope_tab, TreeDesc tree, PosDesc pos, int T_, int d,
                          int dh, size_t row_stride, size_t head_stride, int S_cap, int rope_pos) {
  const int m = blockIdx.x, r = m / T_, t = m % T_;
  int slot, img;
  token_pos(pos, tree, r, t, &slot, &img);
  const int half = dh >> 1, np = dh >> 2;
  int gr = 0, gc = 0;
  if (img >= 0) { gr = min(img / pos.grid_w, rope_pos - 1); gc = img % pos.grid_w; }
  const bool in_cache = slot >= 0 && slot < S_cap;
  const size_t n3 = (size_t)3 * d;
  for (int i = blockIdx.y * blockDim.x + threadIdx.x; i < (d >> 1); i += gridDim.y * blockDim.x) {   // one pair per thread
    const int e0 = 2 * i, hd = e0 / dh, e = e0 % dh;
    const int seg = e / half, ip = (e % half) >> 1;
    float cs = 1.f, sn = 0.f;
    if (img >= 0) {
      const int pv = seg ? gc : gr;
      cs = rope_tab[((size_t)pv * np + ip) * 2];
      sn = rope_tab[((size_t)pv * np + ip) * 2 + 1];
    }
    float v[6] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < splits; ++s) {
      const float* row = qkv + s * split_stride + (size_t)m * n3;
      v[0] += row[e0]; v[1] += row[e0 + 1];
      v[2] += row[d + e0]; v[3] += row[d + e0 + 1];
      v[4] += row[2 * d + e0]; v[5] += row[2 * d + e0 + 1];
    }
    st(q + (size_t)m * d + e0, v[0] * cs - v[1] * sn);
    st(q + (size_t)m * d + e0 + 1, v[0] * sn + v[1] * cs);
    if (in_cache) {
      const size_t hb = (size_t)r * row_stride + (size_t)hd * head_stride;
      st(kc + hb + k_index(slot, e, dh), v[2] * cs - v[3] * sn);
      st(kc + hb + k_index(slot, e + 1, dh), v[2] * sn + v[3] * cs);
      st(vc + hb + v_index(slot, e, dh), v[4]);
      st(vc + hb + v_index(slot, e + 1, dh), v[5]);
    }
  }
}

// ------------------------------------------------------------------------------------------------ attention, one query per workgroup
template <typename T>
__global__ void k_attn_simple(const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc, T* __restrict__ out,
                              TreeDesc tree, PosDesc pos, int T_, int d, int dh, size_t row_stride, size_t head_stride, int S_cap) {
  extern __shared__ float sc[];          // [S_cap] scores, then 16 floats for reductions
  float* red = sc + S_cap;
  const int t = blockIdx.x, hd = blockIdx.y, r = blockIdx.z, m = r * T_ + t;
  const int S = pos.kv_len ? pos.kv_len[r >> 1] : pos.kv_base;
  const int n = min(S + T_, S_cap);
  const uint64_t mask = tree.anc[t];
  const T* qv = q + (size_t)m * d + (size_t)hd * dh;
  const T* kb = kc + (size_t)r * row_stride + (size_t)hd * head_stride;
  const T* vb = vc + (size_t)r * row_stride + (size_t)hd * head_stride;
  const float scale = 1.0f / sqrtf((float)dh);
  float mx = -INFINITY;
  for (int k = threadIdx.x; k < n; k += blockDim.x) {
    bool vis = k < S || ((mask >> (k - S)) & 1ull);
    float sv = -INFINITY;
    if (vis) {
      float dot = 0.f;
      for (int e = 0; e < dh; ++e) dot += ld(qv + e) * ld(kb + k_index(k, e, dh));
      sv = dot * scale;
    }
    sc[k] = sv;
    mx = fmaxf(mx, sv);
  }
  mx = block_max(mx, red);
  float sum = 0.f;
  for (int k = threadIdx.x; k < n; k += blockDim.x) {
    float e = sc[k] == -INFINITY ? 0.f : expf(sc[k] - mx);
    sc[k] = e;
    sum += e;
  }
  sum = block_sum(sum, red);
  for (int e = threadIdx.x; e < dh; e += blockDim.x) {
    float o = 0.f;
    for (int k = 0; k < n; ++k) o += sc[k] * ld(vb + v_index(k, e, dh));
    st(out + (size_t)m * d + (size_t)hd * dh + e, o / sum);
  }
}

// ------------------------------------------------------------------------------------------------ SwiGLU
template <typename T>
__global__ void k_swiglu(const float* __restrict__ gu, int splits, size_t split_stride, T* __restrict__ act, int M, int F,
                         int interleaved) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // one thread per 8 consecutive f
  const int per_row = F >> 3;
  if (i >= (size_t)M * per_row) return;
  const int m = (int)(i / per_row), f0 = (int)(i % per_row) * 8;
  float g[8], u[8], v[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) g[k] = u[k] = 0.f;
  for (int s = 0; s < splits; ++s) {
    const float* row = gu + s * split_stride + (size_t)m * 2 * F;
    // column of gate unit f: f (then up at F + f), or interleaved in blocks of 32: (f/32)*64 + f%32 (up 32 further)
    const int gc = interleaved ? (f0 >> 5) * 64 + (f0 & 31) : f0, uc = interleaved ? gc + 32 : F + f0;
#pragma unroll
    for (int k = 0; k < 8; ++k) { g[k] += row[gc + k]; u[k] += row[uc + k]; }
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) v[k] = g[k] / (1.0f + expf(-g[k])) * u[k];
  store8(act, m, f0, F, v);
}

// ------------------------------------------------------------------------------------------------ GEMM, one wave per output column
// C[m][n] = sum_k A[m][k] * W[n][k]; lanes stride over k (coalesced), 8 rows of A per pass.
template <typename T>
__global__ void k_gemm_simple(const T* __restrict__ A, const T* __restrict__ W, float* __restrict__ C, int M, int N, int K) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 4 + wave, m0 = blockIdx.y * 8;
  if (n >= N) return;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int k = lane; k < K; k += 64) {
    const float w = ld(W + (size_t)n * K + k);
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (m0 + i < M) acc[i] += ld(A + (size_t)(m0 + i) * K + k) * w;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float v = wave_sum(acc[i]);
    if (lane == 0 && m0 + i < M) C[(size_t)(m0 + i) * N + n] = v;
  }
}

// C[splits][M][N] (fp32 partial sums) = A[M][K] * W[N][K]^T (bf16: both operands in packed fragment order)
static int run_gemm(Ctx* c, const void* A, const void* W, float* C, int M, int N, int K, bool allow_split, hipStream_t s) {
  GemmPlan p = plan_gemm(c, M, N, K);
  if (!allow_split) p.splits = 1;
  Timed timed(c, VVS_K_GEMM, s);
  if (c->cfg.dtype == VVS_BF16) {
    mfma_gemm((const bf16_t*)A, (const bf16_t*)W, C, M, N, K, p, s);
    return p.splits;
  }
  dim3 grid((N + 3) / 4, (M + 7) / 8);
  hipLaunchKernelGGL(k_gemm_simple<float>, grid, dim3(256), 0, s, (const float*)A, (const float*)W, C, M, N, K);
  return 1;
}

// ------------------------------------------------------------------------------------------------ one forward over T tokens per row
// bf16, enough rows that no projection needs a grid-level K split: 5 kernels per layer.  The residual
// stream is kept three ways by whoever updates it (embedding kernel, O / down epilogues): fp32 x,
// bf16(x * g) in packed operand order (g = gain of the norm that reads it next), and per-row sums of
// squares; the projections that follow a norm take bf16(x * g) as operand and apply the RMSNorm row
// factor to their output tile.  The packed weights are the caller's bf16 values, unchanged.
static void forward_fused(Ctx* c, const TreeDesc& tree, const PosDesc& pos, int Tq, const int32_t* d_tokens_bt, const void* pc,
                          const void* pu, int chunk_start, const int32_t* forced, int n_forced, int logits_mode, hipStream_t s,
                          bool from_din) {
  const int d = c->d, F = c->F, M = c->R * Tq, NS = (d / 64 + 3) & ~3;   // slabs per row, padded to a multiple of 4 (zeros)
  float* x = (float*)(c->ws + c->w.x);
  bf16_t* xb = (bf16_t*)(c->ws + c->w.h);
  float* ss = (float*)(c->ws + c->w.ss);
  bf16_t* attn = (bf16_t*)(c->ws + c->w.attn);
  bf16_t* act = (bf16_t*)(c->ws + c->w.act);
  EmbedArgs ea{Tq, d, c->V, d_tokens_bt ? 0 : 1, d_tokens_bt, pc, pu, c->cfg.prefix_kind, c->cfg.n_classes, c->P, chunk_start,
               n_forced, forced};
  const float* g_first = (const float*)(c->pw + c->p.layer0 + c->p.g1);   // gain of the first layer's first norm
  const float* gf = (const float*)(c->pw + c->p.gf);
  // verify calls of up to 64 tokens per row at head size 64: projection + attention in one launch, fed by the row-padded operand layout
  const int pad = mfma_qkv_attention_rows(c, pos, Tq);
  const bool qa = pad > 0;
  const int pad_T = qa ? Tq : 0;
  if (from_din) {             // drafter: x = [embedding ; feature] W_fc, through the residual epilogue on a zeroed x
    launch_fill_zero(x, sizeof(float) * (size_t)M * d, s);
    Timed timed(c, VVS_K_GEMM, s);
    mfma_gemm_resid(c, (const bf16_t*)(c->ws + c->w.din), (const bf16_t*)(c->pw + c->p.fc), x, xb, ss, g_first, M, 2 * d, s, pad_T, pad);
  } else {
    Timed timed(c, VVS_K_ELEMENTWISE, s);
    hipLaunchKernelGGL(k_embed_packed, dim3(M), dim3(256), 0, s, x, xb, ss, NS, (const bf16_t*)(c->pw + c->p.embed),
                       (const bf16_t*)(c->pw + c->p.prefix_embed), g_first, ea, pad_T, pad);
  }
  const GemmPlan pq = plan_gemm(c, M, 3 * d, d), pg = plan_gemm(c, M, 2 * F, d);
  for (int l = 0; l < c->L; ++l) {
    const char* lw = c->pw + c->p.layer0 + c->p.layer_stride * l;
    if (qa) {
      Timed timed(c, VVS_K_GEMM, s);
      mfma_qkv_attention(c, l, xb, (const bf16_t*)(lw + c->p.wqkv), ss, tree, pos, Tq, s);
    } else {
      { Timed timed(c, VVS_K_GEMM, s);
        mfma_gemm_qkv(c, l, xb, (const bf16_t*)(lw + c->p.wqkv), ss, tree, pos, Tq, pq, s);
      }
      { Timed timed(c, VVS_K_ATTENTION, s);
        mfma_attention(c, l, tree, pos, Tq, s);
      }
    }
    { Timed timed(c, VVS_K_GEMM, s);
      mfma_gemm_resid(c, attn, (const bf16_t*)(lw + c->p.wo), x, xb, ss, (const float*)(lw + c->p.g2), M, d, s);
    }
    { Timed timed(c, VVS_K_GEMM, s);
      mfma_gemm_swiglu(c, xb, (const bf16_t*)(lw + c->p.wgu), act, ss, M, F, d, pg, s);
    }
    { Timed timed(c, VVS_K_GEMM, s);
      // the next reader of x is the next layer's first norm, or the final norm
      const float* g_next = l + 1 < c->L ? (const float*)(lw + c->p.layer_stride + c->p.g1) : gf;
      mfma_gemm_resid(c, act, (const bf16_t*)(lw + c->p.wd), x, xb, ss, g_next, M, F, s, l + 1 < c->L ? pad_T : 0, pad);
    }
  }
  if (logits_mode == 0) return;
  float* logits = (float*)(c->ws + c->w.logits);
  const bf16_t* wout = (const bf16_t*)(c->pw + c->p.wout);
  if (logits_mode == 1) {
    Timed timed(c, VVS_K_GEMM, s);
    mfma_gemm_scaled(c, xb, wout, logits, ss, M, c->veff, d, plan_gemm(c, M, c->veff, d), s);
  } else {                    // last token of every row
    bf16_t* hf = (bf16_t*)(c->ws + c->w.hf);
    float* ss2 = (float*)(c->ws + c->w.ss2);
    { Timed timed(c, VVS_K_ELEMENTWISE, s);
      hipLaunchKernelGGL(k_gather_rows, dim3(c->R), dim3(256), 0, s, x, ss, gf, hf, ss2, d, NS, Tq, Tq - 1);
    }
    Timed timed(c, VVS_K_GEMM, s);
    mfma_gemm_scaled(c, hf, wout, logits, ss2, c->R, c->veff, d, plan_gemm(c, c->R, c->veff, d), s);
  }
}

template <typename T>
static void forward_t(Ctx* c, const TreeDesc& tree, const PosDesc& pos, int Tq, const int32_t* d_tokens_bt, const void* pc,
                      const void* pu, int chunk_start, const int32_t* forced, int n_forced, int logits_mode, hipStream_t s,
                      bool from_din) {
  const int d = c->d, F = c->F, M = c->R * Tq;
  if (plan_fused(c, M)) {
    forward_fused(c, tree, pos, Tq, d_tokens_bt, pc, pu, chunk_start, forced, n_forced, logits_mode, s, from_din);
    return;
  }
  float* x = (float*)(c->ws + c->w.x);
  T* h = (T*)(c->ws + c->w.h);
  float* go = (float*)(c->ws + c->w.gemm_out);
  T* q = (T*)(c->ws + c->w.q);
  T* attn = (T*)(c->ws + c->w.attn);
  T* act = (T*)(c->ws + c->w.act);
  const float* rope = (const float*)(c->ws + c->w.rope_tab);
  EmbedArgs ea{Tq, d, c->V, d_tokens_bt ? 0 : 1, d_tokens_bt, pc, pu, c->cfg.prefix_kind, c->cfg.n_classes, c->P, chunk_start,
               n_forced, forced};
  int splits = 0;   // partial sums waiting to be added to x
  size_t sstride = 0;
  if (from_din) {             // drafter: x = 0 + [embedding ; feature] W_fc, added by the first norm kernel
    launch_fill_zero(x, sizeof(float) * (size_t)M * d, s);
    splits = run_gemm(c, c->ws + c->w.din, c->pw + c->p.fc, go, M, d, 2 * d, true, s);
    sstride = (size_t)M * d;
  } else {
    Timed timed(c, VVS_K_ELEMENTWISE, s);
    hipLaunchKernelGGL(k_embed<T>, dim3(M), dim3(256), 0, s, x, (const T*)(c->pw + c->p.embed),
                       (const T*)(c->pw + c->p.prefix_embed), ea);
  }
  for (int l = 0; l < c->L; ++l) {
    const char* lw = c->pw + c->p.layer0 + c->p.layer_stride * l;
    T* kc = (T*)c->kv + c->kv_layer_stride * l;
    T* vc = (T*)c->kv + c->kv_v_off + c->kv_layer_stride * l;
    { Timed timed(c, VVS_K_ELEMENTWISE, s);
    launch_add_rmsnorm<T>(M, x, go, splits, sstride, d, (const float*)(lw + c->p.g1), c->cfg.rms_eps, h, 1, 0, s);
    }
    int sp;
    GemmPlan pq = plan_gemm(c, M, 3 * d, d);
    // with 160+ tiles an unsplit projection streams its weights as fast as a split one, and its epilogue
    // does the rotary embedding and the cache write: one kernel less
    if (pq.splits > 1 && ((M + pq.bm - 1) / pq.bm) * (3 * d / pq.bn) >= 160) pq.splits = 1;
    if (c->cfg.dtype == VVS_BF16 && pq.splits == 1) {
      Timed timed(c, VVS_K_GEMM, s);           // projection + rotary + cache write in one kernel
      mfma_gemm_qkv(c, l, (const bf16_t*)h, (const bf16_t*)(lw + c->p.wqkv), nullptr, tree, pos, Tq, pq, s);
    } else {
      sp = run_gemm(c, h, lw + c->p.wqkv, go, M, 3 * d, d, true, s);
      Timed timed(c, VVS_K_ELEMENTWISE, s);
      hipLaunchKernelGGL(k_rope_kv<T>, dim3(M, ((d >> 1) + 255) / 256), dim3(256), 0, s, go, sp, (size_t)M * 3 * d, q, kc, vc, rope, tree, pos, Tq, d, c->dh,
                         c->kv_row_stride, c->kv_head_stride, c->S_cap, c->rope_pos);
    }
    if (c->cfg.dtype == VVS_BF16) {
      Timed timed(c, VVS_K_ATTENTION, s);
      mfma_attention(c, l, tree, pos, Tq, s);
    } else {
      Timed timed(c, VVS_K_ATTENTION, s);
      size_t lds = sizeof(float) * (c->S_cap + 16);
      hipLaunchKernelGGL(k_attn_simple<T>, dim3(Tq, c->H, c->R), dim3(256), lds, s, q, kc, vc, attn, tree, pos, Tq, d, c->dh,
                         c->kv_row_stride, c->kv_head_stride, c->S_cap);
    }
    sp = run_gemm(c, attn, lw + c->p.wo, go, M, d, d, true, s);
    { Timed timed(c, VVS_K_ELEMENTWISE, s);
    launch_add_rmsnorm<T>(M, x, go, sp, (size_t)M * d, d, (const float*)(lw + c->p.g2), c->cfg.rms_eps, h, 1, 0, s);
    }
    GemmPlan pg = plan_gemm(c, M, 2 * F, d);
    if (c->cfg.dtype == VVS_BF16 && pg.splits == 1) {
      Timed timed(c, VVS_K_GEMM, s);           // projection + SwiGLU in one kernel
      mfma_gemm_swiglu(c, (const bf16_t*)h, (const bf16_t*)(lw + c->p.wgu), (bf16_t*)act, nullptr, M, F, d, pg, s);
    } else {
      sp = run_gemm(c, h, lw + c->p.wgu, go, M, 2 * F, d, true, s);
      size_t n = (size_t)M * (F / 8);
      Timed timed(c, VVS_K_ELEMENTWISE, s);
      hipLaunchKernelGGL(k_swiglu<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, go, sp, (size_t)M * 2 * F, act, M, F,
                         c->cfg.dtype == VVS_BF16 ? 1 : 0);
    }
    splits = run_gemm(c, act, lw + c->p.wd, go, M, d, F, true, s);
    sstride = (size_t)M * d;
  }
  if (logits_mode == 0) return;
  T* hf = (T*)(c->ws + c->w.hf);
  float* logits = (float*)(c->ws + c->w.logits);
  const float* gf = (const float*)(c->pw + c->p.gf);
  int Ml;
  if (logits_mode == 1) {     // every token
    Ml = M;
    { Timed timed(c, VVS_K_ELEMENTWISE, s);
    launch_add_rmsnorm<T>(Ml, x, go, splits, sstride, d, gf, c->cfg.rms_eps, hf, 1, 0, s);
    }
  } else {                    // last token of every row
    Ml = c->R;
    { Timed timed(c, VVS_K_ELEMENTWISE, s);
    launch_add_rmsnorm<T>(Ml, x, go, splits, sstride, d, gf, c->cfg.rms_eps, hf, Tq, Tq - 1, s);
    }
  }
  run_gemm(c, hf, c->pw + c->p.wout, logits, Ml, c->veff, d, false, s);
}

void launch_forward(Ctx* c, const TreeDesc& tree, const PosDesc& pos, int T, const int32_t* d_tokens_bt, const void* pc,
                    const void* pu, int chunk_start, const int32_t* forced, int n_forced, int logits_mode, hipStream_t s, bool from_din) {
  if (c->cfg.dtype == VVS_BF16)
    forward_t<bf16_t>(c, tree, pos, T, d_tokens_bt, pc, pu, chunk_start, forced, n_forced, logits_mode, s, from_din);
  else forward_t<float>(c, tree, pos, T, d_tokens_bt, pc, pu, chunk_start, forced, n_forced, logits_mode, s, from_din);
}

// ------------------------------------------------------------------------------------------------ KV commit
// Slot S + path[i] moves to slot S + i for the accepted positions i = 1..a.  path is strictly
// increasing with path[i] >= i, so a destination is never a source of a later position.  A thread
// owns either one chunk (CT: 16 bytes, or one element when the head size does not allow that) of a K
// row or one V element of a head for every accepted position; it reads the sources of up to 8
// positions before it writes them, which leaves one memory round trip per 8 positions.
template <typename T, typename CT>
__global__ __launch_bounds__(256) void k_commit_kv(T* __restrict__ kcache, T* __restrict__ vcache, const int32_t* __restrict__ kv_len,
                                                   const int32_t* __restrict__ accept_len, const int32_t* __restrict__ next_token,
                                                   const int32_t* __restrict__ path, int H, int dh, size_t layer_stride,
                                                   size_t row_stride, size_t head_stride, int S_cap) {
  constexpr int CH = sizeof(CT) / sizeof(T);   // elements per K chunk
  __shared__ int s_src[VVS_MAX_T];
  const int r = blockIdx.x, l = blockIdx.y, b = r >> 1;
  if (next_token[b] < 0) return;
  const int S = kv_len[b], a = accept_len[b];
  if (threadIdx.x < VVS_MAX_T) s_src[threadIdx.x] = path[b * VVS_MAX_T + threadIdx.x];
  __syncthreads();
  T* kb = kcache + l * layer_stride + r * row_stride;
  T* vb = vcache + l * layer_stride + r * row_stride;
  const int n_k = H * dh / CH, n_v = H * dh;
  for (int item = blockIdx.z * blockDim.x + threadIdx.x; item < n_k + n_v; item += gridDim.z * blockDim.x) {   // one item per thread
    if (item < n_k) {
      const int col = item * CH, hd = col / dh, e = col % dh;
      T* kh = kb + hd * head_stride;
      for (int i0 = 1; i0 <= a; i0 += 8) {
        CT tmp[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int i = min(i0 + k, a);
          tmp[k] = *(const CT*)(kh + k_index(min(S + s_src[i], S_cap - 1), e, dh));
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int i = i0 + k;
          if (i <= a && s_src[i] != i && S + s_src[i] < S_cap) *(CT*)(kh + k_index(S + i, e, dh)) = tmp[k];
        }
      }
    } else {
      const int col = item - n_k, hd = col / dh, e = col % dh;
      T* vh = vb + hd * head_stride;
      for (int i0 = 1; i0 <= a; i0 += 8) {
        T tmp[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int i = min(i0 + k, a);
          tmp[k] = vh[v_index(min(S + s_src[i], S_cap - 1), e, dh)];
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int i = i0 + k;
          if (i <= a && s_src[i] != i && S + s_src[i] < S_cap) vh[v_index(S + i, e, dh)] = tmp[k];
        }
      }
    }
  }
}

__global__ void k_commit_state(int32_t* __restrict__ state, int32_t* __restrict__ ring_state, int slots,
                               const int32_t* __restrict__ accept_len, const int32_t* __restrict__ next_token, int B) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B || next_token[b] < 0) return;
  const int n = accept_len[b] + 1;
  state[b] += n;                           // cached length
  state[B + b] += n;                       // emitted image tokens
  state[2 * B + b] = next_token[b];        // pending token
  if (slots > 0) {                         // the feature rings of both rows took n more entries
    const int R = 2 * B;
    for (int r = 2 * b; r < 2 * b + 2; ++r) {
      const int held = ring_state[r], oldest = ring_state[R + r], now = min(held + n, slots);
      ring_state[r] = now;
      ring_state[R + r] = (oldest + held + n - now) % slots;
    }
  }
}

static void launch_push_features(Ctx* c, const int32_t* path, int Tq, int fixed_node, hipStream_t s);

void launch_commit(Ctx* c, hipStream_t s) {
  Timed timed(c, VVS_K_COMMIT, s);
  int32_t* state = (int32_t*)(c->ws + c->w.state);
  const int32_t* oc = (const int32_t*)(c->ws + c->w.outcome);
  const int32_t* accept_len = oc;
  const int32_t* next_token = oc + c->B;
  const int32_t* path = oc + 2 * c->B;
  const bool vec = (c->dh * c->esz) % 16 == 0;
  const int items = c->H * c->dh / (vec ? 16 / (int)c->esz : 1) + c->H * c->dh;   // K chunks + V elements per (row, layer)
  dim3 grid(c->R, c->L, (items + 255) / 256);
  if (c->cfg.dtype == VVS_BF16 && vec)
    hipLaunchKernelGGL((k_commit_kv<bf16_t, uint4>), grid, dim3(256), 0, s, (bf16_t*)c->kv, (bf16_t*)c->kv + c->kv_v_off, state, accept_len,
                       next_token, path, c->H, c->dh, c->kv_layer_stride, c->kv_row_stride, c->kv_head_stride, c->S_cap);
  else if (c->cfg.dtype == VVS_BF16)
    hipLaunchKernelGGL((k_commit_kv<bf16_t, bf16_t>), grid, dim3(256), 0, s, (bf16_t*)c->kv, (bf16_t*)c->kv + c->kv_v_off, state, accept_len,
                       next_token, path, c->H, c->dh, c->kv_layer_stride, c->kv_row_stride, c->kv_head_stride, c->S_cap);
  else if (vec)
    hipLaunchKernelGGL((k_commit_kv<float, uint4>), grid, dim3(256), 0, s, (float*)c->kv, (float*)c->kv + c->kv_v_off, state, accept_len,
                       next_token, path, c->H, c->dh, c->kv_layer_stride, c->kv_row_stride, c->kv_head_stride, c->S_cap);
  else
    hipLaunchKernelGGL((k_commit_kv<float, float>), grid, dim3(256), 0, s, (float*)c->kv, (float*)c->kv + c->kv_v_off, state, accept_len,
                       next_token, path, c->H, c->dh, c->kv_layer_stride, c->kv_row_stride, c->kv_head_stride, c->S_cap);
  launch_push_features(c, path, c->last_T, -1, s);
  hipLaunchKernelGGL(k_commit_state, dim3((c->B + 63) / 64), dim3(64), 0, s, state, (int32_t*)(c->ws + c->w.ring_state),
                     c->cfg.feature_slots, accept_len, next_token, c->B);
}

// ------------------------------------------------------------------------------------------------ token-level feature cache
// Section 4.3 / Algorithm 2 "UpdateCache".  The features of n tokens of the last forward (rows
// r * Tq + node of the residual stream x) are appended to the ring of row r: a feature is
// rmsnorm(x) * gf - the input of the output head - or x itself (pre_norm), stored like an activation
// of the model.  Ring state per row: (entries held, slot of the oldest); the token appended as the
// k-th since the oldest goes to slot (oldest + held + k) % slots.  One workgroup per (row, appended
// token); only the last `slots` tokens of a push are written (older ones would be overwritten by it).
//   path != nullptr: commit - the tokens are path[b][0 .. accept_len[b]] (skipped for finished prompts);
//                    the ring state is advanced afterwards by k_commit_state;
//   path == nullptr: prefill - the single token fixed_node into an emptied ring (state written here).
template <typename T>
__global__ __launch_bounds__(256) void k_push_features(const float* __restrict__ x, const float* __restrict__ gf, T* __restrict__ ring,
                                                       int32_t* __restrict__ ring_state, const int32_t* __restrict__ accept_len,
                                                       const int32_t* __restrict__ next_token, const int32_t* __restrict__ path, int Tq,
                                                       int fixed_node, int R, int d, int slots, int pre_norm, float eps) {
  __shared__ float red[16];
  const int r = blockIdx.x, b = r >> 1;
  int n = 1, held = 0, oldest = 0;
  if (path) {
    if (next_token[b] < 0) return;
    n = accept_len[b] + 1;
    held = ring_state[r];
    oldest = ring_state[R + r];
  }
  const int i = max(0, n - slots) + blockIdx.y;
  if (i >= n) return;
  const int node = path ? path[b * VVS_MAX_T + i] : fixed_node;
  const float* xr = x + ((size_t)r * Tq + node) * d;
  float scale = 1.f;
  if (!pre_norm) {
    float ss = 0.f;
    for (int k = threadIdx.x; k < d; k += blockDim.x) ss += xr[k] * xr[k];
    ss = block_sum(ss, red);
    scale = 1.0f / sqrtf(ss / (float)d + eps);
  }
  T* dst = ring + ((size_t)r * slots + (oldest + held + i) % slots) * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) st(dst + k, pre_norm ? xr[k] : xr[k] * scale * gf[k]);
  if (!path && threadIdx.x == 0) {
    ring_state[r] = 1;
    ring_state[R + r] = 0;
  }
}

static void launch_push_features(Ctx* c, const int32_t* path, int Tq, int fixed_node, hipStream_t s) {
  if (c->cfg.feature_slots < 1) return;
  const int32_t* oc = (const int32_t*)(c->ws + c->w.outcome);
  const float* x = (const float*)(c->ws + c->w.x);
  const float* gf = (const float*)(c->pw + c->p.gf);
  int32_t* rstate = (int32_t*)(c->ws + c->w.ring_state);
  dim3 grid(c->R, path ? c->cfg.feature_slots : 1);
  if (c->cfg.dtype == VVS_BF16)
    hipLaunchKernelGGL(k_push_features<bf16_t>, grid, dim3(256), 0, s, x, gf, (bf16_t*)(c->ws + c->w.ring), rstate, oc, oc + c->B, path,
                       Tq, fixed_node, c->R, c->d, c->cfg.feature_slots, c->cfg.feature_pre_norm, c->cfg.rms_eps);
  else
    hipLaunchKernelGGL(k_push_features<float>, grid, dim3(256), 0, s, x, gf, (float*)(c->ws + c->w.ring), rstate, oc, oc + c->B, path,
                       Tq, fixed_node, c->R, c->d, c->cfg.feature_slots, c->cfg.feature_pre_norm, c->cfg.rms_eps);
}

void launch_push_prefill_feature(Ctx* c, int T_last_chunk, hipStream_t s) {
  launch_push_features(c, nullptr, T_last_chunk, T_last_chunk - 1, s);
}

template <typename T>
__global__ void k_read_features(const T* __restrict__ ring, const int32_t* __restrict__ ring_state, float* __restrict__ out,
                                int32_t* __restrict__ count, int R, int d, int slots) {
  const int r = blockIdx.x, j = blockIdx.y;                // j-th oldest entry of row r
  const int held = ring_state[r], oldest = ring_state[R + r];
  if (j == 0 && threadIdx.x == 0 && (r & 1) == 0) count[r >> 1] = held;
  const T* src = ring + ((size_t)r * slots + (oldest + j) % slots) * d;
  float* dst = out + ((size_t)r * slots + j) * d;
  for (int k = threadIdx.x; k < d; k += blockDim.x) dst[k] = j < held ? ld(src + k) : 0.f;
}

void launch_read_features(Ctx* c, float* d_features, int32_t* d_count, hipStream_t s) {
  const int32_t* rstate = (const int32_t*)(c->ws + c->w.ring_state);
  dim3 grid(c->R, c->cfg.feature_slots);
  if (c->cfg.dtype == VVS_BF16)
    hipLaunchKernelGGL(k_read_features<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)(c->ws + c->w.ring), rstate, d_features, d_count, c->R,
                       c->d, c->cfg.feature_slots);
  else
    hipLaunchKernelGGL(k_read_features<float>, grid, dim3(256), 0, s, (const float*)(c->ws + c->w.ring), rstate, d_features, d_count, c->R,
                       c->d, c->cfg.feature_slots);
}

__global__ void k_read_state(const int32_t* __restrict__ state, int32_t* __restrict__ out, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = state[i];
}

void launch_read_state(Ctx* c, int32_t* d_state, hipStream_t s) {
  int n = 3 * c->B;
  hipLaunchKernelGGL(k_read_state, dim3((n + 255) / 256), dim3(256), 0, s, (const int32_t*)(c->ws + c->w.state), d_state, n);
}

void launch_set_state(Ctx* c, const int32_t* d_state, hipStream_t s) {
  int n = 3 * c->B;
  hipLaunchKernelGGL(k_read_state, dim3((n + 255) / 256), dim3(256), 0, s, d_state, (int32_t*)(c->ws + c->w.state), n);
}

// ------------------------------------------------------------------------------------------------ inspection
__global__ void k_debug_logits(const float* __restrict__ logits, const float* __restrict__ probs_ws, float* __restrict__ raw,
                               float* __restrict__ mixed, float* __restrict__ probs, int B, int T, int veff, float scale) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t per = (size_t)T * veff, n = (size_t)B * per;
  if (i >= n) return;
  const size_t b = i / per, rem = i % per;
  const float lc = logits[(2 * b) * per + rem], lu = logits[(2 * b + 1) * per + rem];
  if (raw) { raw[(2 * b) * per + rem] = lc; raw[(2 * b + 1) * per + rem] = lu; }
  if (mixed) mixed[i] = lu + scale * (lc - lu);
  if (probs) probs[i] = probs_ws[i];
}

void launch_debug_logits(Ctx* c, float* raw, float* mixed, float* probs, hipStream_t s) {
  size_t n = (size_t)c->B * c->last_T * c->veff;
  hipLaunchKernelGGL(k_debug_logits, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float*)(c->ws + c->w.logits),
                     (const float*)(c->ws + c->w.probs), raw, mixed, probs, c->B, c->last_T, c->veff, c->cfg.cfg_scale);
}

template <typename T>
__global__ void k_debug_kv(const T* __restrict__ kh, const T* __restrict__ vh, float* __restrict__ dk, float* __restrict__ dv, int n_slots,
                           int H, int dh, size_t head_stride) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t d = (size_t)H * dh;
  if (i >= (size_t)n_slots * d) return;
  const int slot = (int)(i / d), col = (int)(i % d), hd = col / dh, e = col % dh;
  dk[i] = ld(kh + hd * head_stride + k_index(slot, e, dh));
  dv[i] = ld(vh + hd * head_stride + v_index(slot, e, dh));
}

void launch_debug_kv(Ctx* c, int layer, int row, int n_slots, float* dk, float* dv, hipStream_t s) {
  size_t n = (size_t)n_slots * c->d;
  if (!n) return;
  size_t off = c->kv_layer_stride * layer + c->kv_row_stride * row;
  unsigned blocks = (unsigned)((n + 255) / 256);
  if (c->cfg.dtype == VVS_BF16)
    hipLaunchKernelGGL(k_debug_kv<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t*)c->kv + off,
                       (const bf16_t*)c->kv + c->kv_v_off + off, dk, dv, n_slots, c->H, c->dh, c->kv_head_stride);
  else
    hipLaunchKernelGGL(k_debug_kv<float>, dim3(blocks), dim3(256), 0, s, (const float*)c->kv + off,
                       (const float*)c->kv + c->kv_v_off + off, dk, dv, n_slots, c->H, c->dh, c->kv_head_stride);
}

__global__ void k_sum_splits(const float* __restrict__ part, int splits, size_t n, float* __restrict__ out) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = 0.f;
  for (int s = 0; s < splits; ++s) v += part[s * n + i];
  out[i] = v;
}

void launch_debug_gemm(Ctx* c, int m, int n, int k, const void* a, const void* w, void* scratch, float* out, hipStream_t s) {
  char* wt = (char*)scratch;
  char* at = wt + align_up((size_t)n * k * c->esz, 256);
  float* part = (float*)(at + align_up((size_t)align_up(m, 32) * k * c->esz, 256));
  if (c->cfg.dtype == VVS_BF16) {
    transpose_into<bf16_t>(w, wt, k, n, n, 0, s);
    const size_t total = (size_t)((m + 31) >> 5) * (k >> 4) * 64;
    hipLaunchKernelGGL(k_pack_a, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t*)a, (uint4*)at, m, k);
    a = at;
  } else {
    transpose_into<float>(w, wt, k, n, n, 0, s);
  }
  int sp = run_gemm(c, a, wt, part, m, n, k, true, s);
  size_t cnt = (size_t)m * n;
  hipLaunchKernelGGL(k_sum_splits, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, s, part, sp, cnt, out);
}

}  // namespace vvs
