// Device-side helpers shared by the kernel files.
#pragma once
#include "vvs_internal.h"

namespace vvs {

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round to nearest, ties to even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values in one instruction: lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(floatx2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
__device__ __forceinline__ void st(float* p, float v) { *p = v; }
__device__ __forceinline__ void st(bf16_t* p, float v) { *p = f2bf(v); }

// KV cache layout inside one (layer, row, head) region of S_cap * dh elements.  Both halves are kept
// in the operand order of the attention MFMAs (16x16x32: lane l = 16*g + i supplies 8 consecutive
// contraction values of group g for tile row i), so that one wave-wide 16-byte load reads 1 KiB of
// contiguous memory.  A region is a sequence of steps of 32 slots.
//   K (S^T = K Q^T, contraction over dims): step -> 2 tiles t of 16 keys -> dh/32 blocks kd of 32 dims
//     -> [g = dim%32 / 8][i][dim % 8]; slot w of the step is tile t = (w/4)%2, row i = 4*(w/8) + w%4, so
//     that the 8 scores a lane holds after both tiles are 8 consecutive keys.
//   V (O^T = V^T P^T, contraction over keys): step -> dh/16 blocks dt of 16 dims
//     -> [g = w / 8][i = dim % 16][w % 8].
// Head sizes that are not a multiple of 32 (K) / 16 (V) are only served by the plain kernels and use
// [slot][dim] (K) and [step][dim][32 slots] (V).
__device__ __forceinline__ size_t k_index(int slot, int dim, int dh) {
  if (dh & 31) return (size_t)slot * dh + dim;
  const int w = slot & 31, i = ((w >> 3) << 2) | (w & 3), t = (w >> 2) & 1;
  return ((((size_t)((slot >> 5) * 2 + t) * (dh >> 5) + (dim >> 5)) * 4 + ((dim >> 3) & 3)) * 16 + i) * 8 + (dim & 7);
}
__device__ __forceinline__ size_t v_index(int slot, int dim, int dh) {
  if (dh & 15) return ((size_t)(slot >> 5) * dh + dim) * 32 + (slot & 31);
  const int w = slot & 31;
  return ((((size_t)(slot >> 5) * (dh >> 4) + (dim >> 4)) * 4 + (w >> 3)) * 16 + (dim & 15)) * 8 + (w & 7);
}

// GEMM operands of the bf16 path are stored in MFMA fragment order: 1 KiB blocks of 32 rows x 16
// contraction indices; inside a block lane = row%32 + 32*((k%16)/8) holds 8 consecutive k.
__device__ __host__ __forceinline__ size_t pack_index(int row, int k, int K) {
  return ((size_t)(row >> 5) * (K >> 4) + (k >> 4)) * 512 + (size_t)(((row & 31) + 32 * ((k >> 3) & 1)) * 8 + (k & 7));
}
// Stores 8 consecutive activation values (k0 % 8 == 0) of one row: row-major fp32, or one 16-byte
// chunk of the packed bf16 layout.
__device__ __forceinline__ void store8(float* base, int row, int k0, int K, const float* v) {
  float4* p = (float4*)(base + (size_t)row * K + k0);
  p[0] = make_float4(v[0], v[1], v[2], v[3]);
  p[1] = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t* base, int row, int k0, int K, const float* v) {
  uint4 o;
  o.x = pack2bf(v[0], v[1]);
  o.y = pack2bf(v[2], v[3]);
  o.z = pack2bf(v[4], v[5]);
  o.w = pack2bf(v[6], v[7]);
  *(uint4*)(base + pack_index(row, k0, K)) = o;
}

// wave64 reductions, fixed order
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Block reductions over blockDim.x threads (multiple of 64, <= 1024); red = 16 floats of LDS.
// Every thread gets the result; deterministic (fixed tree).
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}
// two sums at once (one pair of barriers); red = 32 floats of LDS
__device__ __forceinline__ float2 block_sum2(float a, float b, float* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {       // the two butterfly chains interleaved: their latencies overlap
    const float ta = __shfl_xor(a, o, 64), tb = __shfl_xor(b, o, 64);
    a += ta;
    b += tb;
  }
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { red[w] = a; red[16 + w] = b; }
  __syncthreads();
  float ta = 0.f, tb = 0.f;
  for (int i = 0; i < nw; ++i) { ta += red[i]; tb += red[16 + i]; }
  return make_float2(ta, tb);
}
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  return t;
}
__device__ __forceinline__ int block_min_int(int v, int* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  int t = red[0];
  for (int i = 1; i < nw; ++i) t = min(t, red[i]);
  return t;
}
__device__ __forceinline__ int block_max_int(int v, int* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, 64));
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  int t = red[0];
  for (int i = 1; i < nw; ++i) t = max(t, red[i]);
  return t;
}

// Position of block token t of row r: cache slot and image-token index (< 0: prefix token).
__device__ __forceinline__ void token_pos(const PosDesc& pos, const TreeDesc& tree, int r, int t, int* slot, int* img) {
  if (pos.kv_len) {
    int b = r >> 1;
    *slot = pos.kv_len[b] + t;
    *img = pos.n_emitted[b] - 1 + tree.depth[t];
  } else {
    *slot = pos.kv_base + t;
    *img = *slot - pos.prefix_len;
  }
}

// A kernel that uses more than 64 KiB of dynamic LDS has to be allowed to, once per device: remembers per
// (kernel, device) that it has been done.  Host code; launches of one context come from one thread at a time.
inline void allow_dynamic_lds(const void* kernel, size_t bytes) {
  struct Done { const void* fn; int dev; };
  static std::vector<Done> done;
  int dev = 0;
  (void)hipGetDevice(&dev);
  for (const Done& d : done)
    if (d.fn == kernel && d.dev == dev) return;
  // a failure shows up as an invalid-configuration error of the launch that follows
  (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  done.push_back(Done{kernel, dev});
}

// MFMA attention / GEMM launchers (vvs_mfma.hip)
void mfma_gemm(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, GemmPlan p, hipStream_t s);
void mfma_gemm_scaled(Ctx* c, const bf16_t* A, const bf16_t* W, float* C, const float* ss, int M, int N, int K, GemmPlan p, hipStream_t s);
void mfma_gemm_resid(Ctx* c, const bf16_t* A, const bf16_t* W, float* x, bf16_t* xb, float* ss_out, const float* g_next, int M, int K,
                     hipStream_t s, int xb_T = 0, int xb_pad = 0 /* xb_T > 0: xb row-padded to xb_pad rows per xb_T tokens */);
int mfma_qkv_attention_rows(const Ctx* c, const PosDesc& pos, int T);
void mfma_qkv_attention(Ctx* c, int layer, const bf16_t* A, const bf16_t* Wqkv, const float* ss, const TreeDesc& tree, const PosDesc& pos,
                        int T, hipStream_t s);
void mfma_gemm_swiglu(Ctx* c, const bf16_t* A, const bf16_t* Wgu, bf16_t* act, const float* ss, int M, int F, int K, GemmPlan p,
                      hipStream_t s);
void mfma_gemm_qkv(Ctx* c, int layer, const bf16_t* A, const bf16_t* Wqkv, const float* ss, const TreeDesc& tree, const PosDesc& pos, int T,
                   GemmPlan p, hipStream_t s);
void mfma_attention(Ctx* c, int layer, const TreeDesc& tree, const PosDesc& pos, int T, hipStream_t s);

}  // namespace vvs
