// bf16 MFMA kernels for gfx950: the GEMM behind the QKV / O / MLP / lm_head projections and the
// tree-masked attention over the KV cache.
//
// MFMA operand layouts used below (wave64):
//   v_mfma_f32_32x32x16_bf16: lane l gives A[i = l%32][8 k-values of group l/32] and
//     B[same 8 k-values][j = l%32]; accumulator register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32].
//   v_mfma_f32_16x16x32_bf16: lane l gives A[i = l%16][8 k-values of group l/16] and
//     B[same 8 k-values][j = l%16]; accumulator register r of lane l is D[4*(l/16) + r][l%16].
// A and B always pair the same (group, element) slot, so only "8 consecutive k per lane" matters.
#include "vvs_device.h"

namespace vvs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// ------------------------------------------------------------------------------------------------ GEMM
// C[split][M][N] (fp32) = A[M][K] (bf16, row-major) * W[N][K]^T (bf16, K contiguous), K range of the
// split.  Workgroup tile BM x BN, 4 waves as 2 x 2, each wave (BM/2) x (BN/2) in 32x32x16 MFMA tiles;
// BK = 64 staged through LDS (row stride 72 elements: conflict-free 16-byte fragment reads), the next
// tile's global loads are in flight while the current one is multiplied.
template <int BM, int BN>
__global__ __launch_bounds__(256) void k_gemm_mfma(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, float* __restrict__ C,
                                                   int M, int N, int K, int kt_per_split) {
  constexpr int BK = 64, LS = BK + 8;
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int AP = BM / 32, BP = BN / 32;
  __shared__ __attribute__((aligned(16))) bf16_t sA[BM * LS];
  __shared__ __attribute__((aligned(16))) bf16_t sB[BN * LS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN, split = blockIdx.z;
  const int kt_total = K / BK;
  const int kt0 = split * kt_per_split, kt1 = min(kt_total, kt0 + kt_per_split);
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  // staging: each thread moves one 16-byte chunk per 32 tile rows (named registers, not arrays, so
  // that they stay in VGPRs)
  const int lrow = tid >> 3, lchunk = tid & 7;
  const bf16_t* pa = A + lchunk * 8;
  const bf16_t* pb = W + (size_t)(n0 + lrow) * K + lchunk * 8;
  const size_t ar0 = (size_t)min(m0 + lrow, M - 1) * K, ar1 = (size_t)min(m0 + 32 + lrow, M - 1) * K;
  const size_t ar2 = (size_t)min(m0 + 64 + lrow, M - 1) * K, ar3 = (size_t)min(m0 + 96 + lrow, M - 1) * K;
  const size_t br = (size_t)32 * K;
  uint4 ra0, ra1, ra2, ra3, rb0, rb1, rb2, rb3;
  ra2 = ra3 = rb2 = rb3 = make_uint4(0, 0, 0, 0);
#define VVS_GLOAD(kt)                                              \
  {                                                                \
    const size_t ko = (size_t)(kt) * BK;                           \
    ra0 = *(const uint4*)(pa + ar0 + ko);                          \
    ra1 = *(const uint4*)(pa + ar1 + ko);                          \
    if (AP > 2) {                                                  \
      ra2 = *(const uint4*)(pa + ar2 + ko);                        \
      ra3 = *(const uint4*)(pa + ar3 + ko);                        \
    }                                                              \
    rb0 = *(const uint4*)(pb + ko);                                \
    rb1 = *(const uint4*)(pb + br + ko);                           \
    if (BP > 2) {                                                  \
      rb2 = *(const uint4*)(pb + 2 * br + ko);                     \
      rb3 = *(const uint4*)(pb + 3 * br + ko);                     \
    }                                                              \
  }
  VVS_GLOAD(min(kt0, kt_total - 1));
  for (int kt = kt0; kt < kt1; ++kt) {
    __syncthreads();
    {
      bf16_t* da = sA + lrow * LS + lchunk * 8;
      bf16_t* db = sB + lrow * LS + lchunk * 8;
      *(uint4*)(da) = ra0;
      *(uint4*)(da + 32 * LS) = ra1;
      if (AP > 2) { *(uint4*)(da + 64 * LS) = ra2; *(uint4*)(da + 96 * LS) = ra3; }
      *(uint4*)(db) = rb0;
      *(uint4*)(db + 32 * LS) = rb1;
      if (BP > 2) { *(uint4*)(db + 64 * LS) = rb2; *(uint4*)(db + 96 * LS) = rb3; }
    }
    __syncthreads();
    VVS_GLOAD(min(kt + 1, kt1 - 1));   // the last iteration re-reads its own tile (no branch around the loads)
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[TM], bfr[TN];
      const int koff = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = as_bf16x8(*(const uint4*)(sA + (wm * (BM / 2) + i * 32 + (lane & 31)) * LS + koff));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = as_bf16x8(*(const uint4*)(sB + (wn * (BN / 2) + j * 32 + (lane & 31)) * LS + koff));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  }
#undef VVS_GLOAD
  float* Cs = C + (size_t)split * M * N;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * (BN / 2) + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * (BM / 2) + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (m < M) Cs[(size_t)m * N + n] = acc[i][j][r];
      }
    }
}

void mfma_gemm(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, GemmPlan p, hipStream_t s) {
  const int kt = K / 64;
  const int per = (kt + p.splits - 1) / p.splits;
  dim3 grid(N / p.bn, (M + p.bm - 1) / p.bm, p.splits);
  if (p.bm == 128 && p.bn == 128) hipLaunchKernelGGL((k_gemm_mfma<128, 128>), grid, dim3(256), 0, s, A, W, C, M, N, K, per);
  else if (p.bm == 64 && p.bn == 128) hipLaunchKernelGGL((k_gemm_mfma<64, 128>), grid, dim3(256), 0, s, A, W, C, M, N, K, per);
  else hipLaunchKernelGGL((k_gemm_mfma<64, 64>), grid, dim3(256), 0, s, A, W, C, M, N, K, per);
}

// ------------------------------------------------------------------------------------------------ attention
// One workgroup per (head, row).  Scores are computed transposed, S^T[key][query] = K * Q^T, so the
// accumulator layout (lane = query, registers = keys) is directly the B operand of
// O^T[dim][query] = V^T[dim][key] * P^T[key][query] and the online-softmax state of a query lives in
// one lane.  K rows ([slot][dim], dim contiguous) and V blocks ([dim][32 slots], slot contiguous) are
// loaded straight from the cache into MFMA operand registers - every key is used by exactly one wave,
// so there is nothing to share through LDS; the 4 waves take 32-key steps round-robin and merge their
// partial (max, sum, O) through LDS at the end.  Only the last T keys (the block itself) are masked.
template <int DH, int NQB>
__global__ __launch_bounds__(256) void k_attn_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc,
                                                   const bf16_t* __restrict__ vc, bf16_t* __restrict__ out, TreeDesc tree,
                                                   PosDesc pos, int T, int d, size_t row_stride, size_t head_stride, float c_exp) {
  constexpr int KD = DH / 32, DT = DH / 16, NQ = NQB * 16;
  __shared__ float s_m[3][NQ], s_l[3][NQ];
  __shared__ float s_o[3][NQ][DH + 1];
  const int hd = blockIdx.x, r = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, ql = lane & 15;
  const int S = pos.kv_len ? pos.kv_len[r >> 1] : pos.kv_base;
  const int n_keys = S + T;
  const int nsteps = (n_keys + 31) >> 5;
  const bf16_t* kb = kc + (size_t)r * row_stride + (size_t)hd * head_stride;
  const bf16_t* vb = vc + (size_t)r * row_stride + (size_t)hd * head_stride;

  bf16x8 qf[NQB][KD];
  uint64_t mask[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int tq = qb * 16 + ql;
    mask[qb] = tq < T ? tree.anc[tq] : 0ull;
#pragma unroll
    for (int kd = 0; kd < KD; ++kd) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (tq < T) v = *(const uint4*)(q + ((size_t)r * T + tq) * d + (size_t)hd * DH + kd * 32 + g * 8);
      qf[qb][kd] = as_bf16x8(v);
    }
  }
  float m_run[NQB], l_run[NQB];
  floatx4 o[NQB][DT];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[qb][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  for (int step = wave; step < nsteps; step += 4) {
    const int key0 = step << 5;
    bf16x8 kf[2][KD], vf[DT];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key = key0 + 8 * (ql >> 2) + 4 * t + (ql & 3);
#pragma unroll
      for (int kd = 0; kd < KD; ++kd) kf[t][kd] = as_bf16x8(*(const uint4*)(kb + (size_t)key * DH + kd * 32 + g * 8));
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      vf[dt] = as_bf16x8(*(const uint4*)(vb + ((size_t)step * DH + dt * 16 + ql) * 32 + g * 8));
    const bool tail = key0 + 32 > S;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      floatx4 s2[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        s2[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kd = 0; kd < KD; ++kd) s2[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][kd], qf[qb][kd], s2[t], 0, 0, 0);
      }
      float sv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) sv[i] = s2[i >> 2][i & 3];
      if (tail) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int key = key0 + 8 * g + i;
          bool vis = key < S;
          if (!vis && key < n_keys) vis = (mask[qb] >> (key - S)) & 1ull;
          if (!vis) sv[i] = -INFINITY;
        }
      }
      float mx = sv[0];
#pragma unroll
      for (int i = 1; i < 8; ++i) mx = fmaxf(mx, sv[i]);
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[qb], mx);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = exp2f((m_run[qb] - m_safe) * c_exp);
      uint32_t pk[4];
      float rs = 0.f;
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        const bf16_t p0 = f2bf(exp2f((sv[i] - m_safe) * c_exp));
        const bf16_t p1 = f2bf(exp2f((sv[i + 1] - m_safe) * c_exp));
        rs += bf2f(p0) + bf2f(p1);
        pk[i >> 1] = (uint32_t)p0 | ((uint32_t)p1 << 16);
      }
      rs += __shfl_xor(rs, 16, 64);
      rs += __shfl_xor(rs, 32, 64);
      l_run[qb] = l_run[qb] * alpha + rs;
      m_run[qb] = m_new;
      const bf16x8 pf = as_bf16x8(make_uint4(pk[0], pk[1], pk[2], pk[3]));
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) o[qb][dt][rr] *= alpha;
        o[qb][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf, o[qb][dt], 0, 0, 0);
      }
    }
  }

  // merge the four waves' partial results (waves 1..3 publish, wave 0 combines and writes)
  if (wave > 0) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int qi = qb * 16 + ql;
      if (g == 0) { s_m[wave - 1][qi] = m_run[qb]; s_l[wave - 1][qi] = l_run[qb]; }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) s_o[wave - 1][qi][dt * 16 + 4 * g + rr] = o[qb][dt][rr];
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int qi = qb * 16 + ql;
      float m = m_run[qb];
#pragma unroll
      for (int w = 0; w < 3; ++w) m = fmaxf(m, s_m[w][qi]);
      const float m_safe = m == -INFINITY ? 0.f : m;
      const float a0 = exp2f((m_run[qb] - m_safe) * c_exp);
      float l = l_run[qb] * a0;
      float aw[3];
#pragma unroll
      for (int w = 0; w < 3; ++w) {
        aw[w] = exp2f((s_m[w][qi] - m_safe) * c_exp);
        l += s_l[w][qi] * aw[w];
      }
      const float inv = 1.0f / l;
      if (qi < T) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          uint32_t pk[2];
#pragma unroll
          for (int rr = 0; rr < 4; rr += 2) {
            float v0 = o[qb][dt][rr] * a0, v1 = o[qb][dt][rr + 1] * a0;
#pragma unroll
            for (int w = 0; w < 3; ++w) {
              v0 += s_o[w][qi][dt * 16 + 4 * g + rr] * aw[w];
              v1 += s_o[w][qi][dt * 16 + 4 * g + rr + 1] * aw[w];
            }
            pk[rr >> 1] = (uint32_t)f2bf(v0 * inv) | ((uint32_t)f2bf(v1 * inv) << 16);
          }
          *(uint2*)(out + ((size_t)r * T + qi) * d + (size_t)hd * DH + dt * 16 + 4 * g) = make_uint2(pk[0], pk[1]);
        }
      }
    }
  }
}

void mfma_attention(Ctx* c, int layer, const TreeDesc& tree, const PosDesc& pos, int T, hipStream_t s) {
  const bf16_t* q = (const bf16_t*)(c->ws + c->w.q);
  bf16_t* out = (bf16_t*)(c->ws + c->w.attn);
  const bf16_t* kc = (const bf16_t*)c->kv + c->kv_layer_stride * layer;
  const bf16_t* vc = (const bf16_t*)c->kv + c->kv_v_off + c->kv_layer_stride * layer;
  const float c_exp = 1.4426950408889634f / sqrtf((float)c->dh);
  dim3 grid(c->H, c->R);
  const int nqb = T <= 16 ? 1 : (T <= 32 ? 2 : 4);
#define VVS_ATTN(DH, NQB)                                                                                             \
  hipLaunchKernelGGL((k_attn_mfma<DH, NQB>), grid, dim3(256), 0, s, q, kc, vc, out, tree, pos, T, c->d, c->kv_row_stride, \
                     c->kv_head_stride, c_exp)
  if (c->dh == 64) {
    if (nqb == 1) VVS_ATTN(64, 1); else if (nqb == 2) VVS_ATTN(64, 2); else VVS_ATTN(64, 4);
  } else {
    if (nqb == 1) VVS_ATTN(128, 1); else VVS_ATTN(128, 2);   // T <= 32 is enforced at context creation for head size 128
  }
#undef VVS_ATTN
}

}  // namespace vvs
