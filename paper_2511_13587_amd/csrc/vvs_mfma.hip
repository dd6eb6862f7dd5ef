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
// C[split][M][N] (fp32) = A[M][K] * W[N][K]^T with both operands pre-packed in MFMA fragment order:
//   block (rb, kb) of a matrix with rows r and contraction index k = 64 lanes x 8 bf16 (1 KiB,
//   contiguous); lane l holds row rb*32 + l%32, k = kb*16 + 8*(l/32) .. +8.        (pack_index)
// A workgroup owns a (TM*32) x (TN*32) output tile.  Its 4 waves split the K range between them and
// each wave streams ITS OWN A and B fragments straight from global memory into MFMA operand
// registers - 1 KiB fully coalesced per load instruction, D k-steps in flight per wave, no LDS and
// no barrier in the main loop (at these sizes a projection is bound by memory latency, not by MFMA
// rate: the whole weight matrix is only a few MB, so what matters is how many bytes every CU keeps
// in flight).  The 4 partial tiles are summed through LDS at the end, in a fixed order.
//
// Epilogues (after the 4-way sum):
//   EPI_PARTIAL: store the fp32 tile to C[split] (consumers add the splits);
//   EPI_SWIGLU : the weight rows are interleaved so that tile columns 0..31 are gate and 32..63 up
//                outputs of the same 32 hidden units: write silu(gate) * up as the packed bf16
//                operand of the down projection (one K split only);
//   EPI_QKV    : the tile lies inside the q, k or v third of the fused projection: apply the 2D
//                rotary embedding to q and k, write q (bf16 row-major) and put k / v into the cache
//                slots of their tokens (one K split only);
//   EPI_RESID  : O / down projection: x += tile (fp32 residual stream, each element owned by one
//                thread), also written as the packed bf16 operand of the next projection, plus the
//                sum of squares of the tile's 64 columns per row (one K split only).
// Row scale: RMSNorm is x * s_m * g with s_m = rsqrt(mean_k x_mk^2 + eps).  The gain g is folded into
// the weights when they are packed, the operand is bf16(x) itself, and s_m - a per-row factor that
// commutes with the contraction - multiplies the accumulated tile in the epilogue; s_m comes from the
// per-64-column sums of squares that the producer of x (EPI_RESID or the embedding kernel) left in ss.
// This removes the separate normalisation pass between two projections.
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_QKV = 2, EPI_RESID = 3 };

struct GemmEpi {
  const float* ss; int NS; float eps; int dnorm;           // row scale (ss == nullptr: no scaling); ss[M][NS]
  bf16_t* act; int F;                                      // EPI_SWIGLU
  float* x; bf16_t* xb; float* ss_out;                     // EPI_RESID
  bf16_t* q; bf16_t* kc; bf16_t* vc; const float* rope;    // EPI_QKV
  int T, d, dh, S_cap, rope_pos;
  size_t row_stride, head_stride;
  PosDesc pos;
  TreeDesc tree;
};

template <int TM, int TN, int D, int EPI>
__global__ __launch_bounds__(256) void k_gemm_direct(const uint4* __restrict__ Ap, const uint4* __restrict__ Wp, float* __restrict__ C,
                                                     int M, int N, int K, int kb_per_split, const GemmEpi ep) {
  constexpr int BM = TM * 32, BN = TN * 32, LDC = BN + 4;
  extern __shared__ float red[];           // [4][BM][LDC]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // XCD-aware tile order.  Workgroups are dealt to the 8 XCDs round-robin by linear id, and each XCD
  // has its own L2.  Column tiles are taken in groups of 8 (one per XCD); inside a group the row
  // tiles of one column tile get ids 8 apart: they run at the same time on the same XCD, so a weight
  // tile is fetched from HBM once and then hits in that XCD's L2.
  const int MT = (M + BM - 1) / BM, NT = N / BN;
  int tile_m, tile_n;
  {
    const int id = blockIdx.x, grp = id / (8 * MT), rem = id % (8 * MT);
    const int cols = min(8, NT - grp * 8);
    tile_m = rem / cols;
    tile_n = grp * 8 + rem % cols;
  }
  __shared__ float rs[BM];                 // per-row RMSNorm factor of this tile's rows (loaded first: hidden behind the main loop)
  if (threadIdx.x < BM * 4) {              // 4 lanes per row, each sums every 4th group of 4 slabs: all loads independent
    const int row = threadIdx.x >> 2, part = threadIdx.x & 3;
    const int m = tile_m * BM + row;
    float t = 0.f;
    if (ep.ss && m < M) {
      const float4* p4 = (const float4*)(ep.ss + (size_t)m * ep.NS);     // rows are padded to a multiple of 4 slabs (zeros)
      const int nq = ep.NS >> 2;
      float4 v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = (part + 4 * i < nq) ? p4[part + 4 * i] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int i = 0; i < 4; ++i) t += (v[i].x + v[i].y) + (v[i].z + v[i].w);
      for (int qd = part + 16; qd < nq; qd += 4) { const float4 w = p4[qd]; t += (w.x + w.y) + (w.z + w.w); }
    }
    t += __shfl_xor(t, 1, 64);
    t += __shfl_xor(t, 2, 64);
    if (part == 0) rs[row] = (ep.ss && m < M) ? 1.0f / sqrtf(t / (float)ep.dnorm + ep.eps) : 1.f;
  }
  const int KB = K >> 4;
  const int s0 = blockIdx.z * kb_per_split, s1 = min(KB, s0 + kb_per_split);
  const int per_w = (max(s1 - s0, 0) + 3) >> 2;
  const int w0 = s0 + wave * per_w, w1 = min(s1, w0 + per_w);
  const int nk = max(w1 - w0, 0);
  const uint4* ap[TM];
  const uint4* bp[TN];
#pragma unroll
  for (int t = 0; t < TM; ++t) ap[t] = Ap + ((size_t)(tile_m * TM + t) * KB) * 64 + lane;
#pragma unroll
  for (int t = 0; t < TN; ++t) bp[t] = Wp + ((size_t)(tile_n * TN + t) * KB) * 64 + lane;
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  uint4 fa[D][TM], fb[D][TN];
#pragma unroll
  for (int i = 0; i < D; ++i) {
    const size_t kk = (size_t)min(w0 + i, KB - 1) * 64;      // clamped: loads past the range are unused
#pragma unroll
    for (int t = 0; t < TM; ++t) fa[i][t] = ap[t][kk];
#pragma unroll
    for (int t = 0; t < TN; ++t) fb[i][t] = bp[t][kk];
    // keep the load groups in program order: the wait before a k-step's MFMAs is then "all but the
    // (D-1) younger groups", never "everything"
    __builtin_amdgcn_sched_barrier(0);
  }
  for (int kb = 0; kb < nk; kb += D) {
#pragma unroll
    for (int i = 0; i < D; ++i) {
      if (kb + i < nk) {
#pragma unroll
        for (int ti = 0; ti < TM; ++ti)
#pragma unroll
          for (int tj = 0; tj < TN; ++tj)
            acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fa[i][ti]), as_bf16x8(fb[i][tj]), acc[ti][tj], 0, 0, 0);
      }
      const size_t kk = (size_t)min(w0 + kb + i + D, KB - 1) * 64;
#pragma unroll
      for (int t = 0; t < TM; ++t) fa[i][t] = ap[t][kk];
#pragma unroll
      for (int t = 0; t < TN; ++t) fb[i][t] = bp[t][kk];
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // publish the partial tile: acc[i][j][r] is row i*32 + 8*(r/4) + 4*(lane/32) + r%4, col j*32 + lane%32
  float* mine = red + (size_t)wave * BM * LDC;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        mine[(i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * LDC + j * 32 + (lane & 31)] = acc[i][j][r];
  __syncthreads();
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  constexpr int PS = BM * LDC;   // stride between the waves' partial tiles
  // sum of the four waves' partial tiles for 4 consecutive columns, fixed order
  auto sum4 = [&](const float* p) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + PS), c = *(const float4*)(p + 2 * PS), d = *(const float4*)(p + 3 * PS);
    return make_float4(((a.x + b.x) + c.x) + d.x, ((a.y + b.y) + c.y) + d.y, ((a.z + b.z) + c.z) + d.z, ((a.w + b.w) + c.w) + d.w);
  };
  if constexpr (EPI == EPI_PARTIAL) {
    float* Cs = C + (size_t)blockIdx.z * M * N;
    for (int u = threadIdx.x; u < BM * (BN / 4); u += 256) {       // one unit = (row, 4 consecutive columns)
      const int row = u / (BN / 4), col = (u % (BN / 4)) * 4;
      if (m0 + row < M) {
        float4 v = sum4(red + row * LDC + col);
        const float sc = rs[row];
        v.x *= sc; v.y *= sc; v.z *= sc; v.w *= sc;
        *(float4*)(Cs + (size_t)(m0 + row) * N + n0 + col) = v;
      }
    }
  } else if constexpr (EPI == EPI_SWIGLU) {
    static_assert(TN % 2 == 0, "gate / up blocks of 32 columns alternate inside the tile");
    for (int u = threadIdx.x; u < BM * (BN / 16); u += 256) {       // one unit = (row, 8 consecutive hidden units)
      const int row = u / (BN / 16), fl = (u % (BN / 16)) * 8;      // fl: hidden unit inside the tile, 0 .. BN/2
      if (m0 + row >= M) continue;
      const float* pg = red + row * LDC + (fl >> 5) * 64 + (fl & 31);
      const float4 g0 = sum4(pg), g1 = sum4(pg + 4), u0 = sum4(pg + 32), u1 = sum4(pg + 36);
      const float gs[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      const float us[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float g = gs[i] * rs[row], up = us[i] * rs[row];
        v[i] = g / (1.0f + expf(-g)) * up;
      }
      store8(ep.act, m0 + row, tile_n * (BN / 2) + fl, ep.F, v);
    }
  } else if constexpr (EPI == EPI_RESID) {
    static_assert(BN == 64, "the sums of squares are kept per 64-column slab");
    for (int u = threadIdx.x; u < BM * 8; u += 256) {              // one unit = (row, 8 consecutive columns); 8 lanes share a row
      const int row = u >> 3, c8 = (u & 7) * 8;
      const int m = m0 + row;
      float sq = 0.f;
      if (m < M) {
        const float4 a = sum4(red + row * LDC + c8), b = sum4(red + row * LDC + c8 + 4);
        float* xp = ep.x + (size_t)m * N + n0 + c8;
        const float4 xa = *(const float4*)xp, xb4 = *(const float4*)(xp + 4);
        float v[8] = {xa.x + a.x, xa.y + a.y, xa.z + a.z, xa.w + a.w, xb4.x + b.x, xb4.y + b.y, xb4.z + b.z, xb4.w + b.w};
        *(float4*)xp = make_float4(v[0], v[1], v[2], v[3]);
        *(float4*)(xp + 4) = make_float4(v[4], v[5], v[6], v[7]);
        store8(ep.xb, m, n0 + c8, N, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) sq += v[i] * v[i];
      }
      sq += __shfl_xor(sq, 1, 64);
      sq += __shfl_xor(sq, 2, 64);
      sq += __shfl_xor(sq, 4, 64);
      if (m < M && c8 == 0) ep.ss_out[(size_t)m * ep.NS + tile_n] = sq;
    }
  } else {
    const int half = ep.dh >> 1, np = ep.dh >> 2;
    for (int u = threadIdx.x; u < BM * (BN / 16); u += 256) {   // one unit = (row, 16 consecutive columns)
      const int row = u / (BN / 16), c0 = (u % (BN / 16)) * 16;
      const int m = m0 + row;
      if (m >= M) continue;
      const float* p = red + row * LDC + c0;
      const float4 s0 = sum4(p), s1 = sum4(p + 4), s2 = sum4(p + 8), s3 = sum4(p + 12);
      float v[16] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w, s2.x, s2.y, s2.z, s2.w, s3.x, s3.y, s3.z, s3.w};
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] *= rs[row];
      const int n = n0 + c0, sec = n / ep.d, eg = n % ep.d, hd = eg / ep.dh, e = eg % ep.dh;
      const int r = m / ep.T, t = m % ep.T;
      int slot, img;
      token_pos(ep.pos, ep.tree, r, t, &slot, &img);
      if (sec < 2 && img >= 0) {
        const int gr = min(img / ep.pos.grid_w, ep.rope_pos - 1), gc = img % ep.pos.grid_w;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const int ei = e + i, pv = (ei / half) ? gc : gr, ip = (ei % half) >> 1;
          const float cs = ep.rope[((size_t)pv * np + ip) * 2], sn = ep.rope[((size_t)pv * np + ip) * 2 + 1];
          const float a = v[i], b = v[i + 1];
          v[i] = a * cs - b * sn;
          v[i + 1] = a * sn + b * cs;
        }
      }
      uint32_t w[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) w[i] = (uint32_t)f2bf(v[2 * i]) | ((uint32_t)f2bf(v[2 * i + 1]) << 16);
      if (sec == 0) {
        uint4* dst = (uint4*)(ep.q + (size_t)m * ep.d + eg);
        dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
        dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
      } else if (slot >= 0 && slot < ep.S_cap) {
        const size_t hb = (size_t)r * ep.row_stride + (size_t)hd * ep.head_stride;
        if (sec == 1) {
          uint4* dst = (uint4*)(ep.kc + hb + (size_t)slot * ep.dh + e);
          dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
          dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i) ep.vc[hb + v_index(slot, e + i, ep.dh)] = (bf16_t)(w[i >> 1] >> ((i & 1) * 16));
        }
      }
    }
  }
}

template <int TM, int TN, int D, int EPI>
static void launch_gemm_direct(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, int splits, const GemmEpi& ep,
                               hipStream_t s) {
  constexpr size_t lds = (size_t)4 * TM * 32 * (TN * 32 + 4) * sizeof(float);
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_direct<TM, TN, D, EPI>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
    configured = true;
  }
  const int KB = K / 16;
  const int per = (KB + splits - 1) / splits;
  dim3 grid((N / (TN * 32)) * ((M + TM * 32 - 1) / (TM * 32)), 1, splits);
  hipLaunchKernelGGL((k_gemm_direct<TM, TN, D, EPI>), grid, dim3(256), lds, s, (const uint4*)A, (const uint4*)W, C, M, N, K, per, ep);
}

template <int EPI>
static void gemm_dispatch(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, GemmPlan p, const GemmEpi& ep, hipStream_t s) {
  if (p.bm == 32) launch_gemm_direct<1, 2, 8, EPI>(A, W, C, M, N, K, p.splits, ep, s);
  else if (p.bn == 128) launch_gemm_direct<2, 4, 4, EPI>(A, W, C, M, N, K, p.splits, ep, s);
  else launch_gemm_direct<2, 2, 6, EPI>(A, W, C, M, N, K, p.splits, ep, s);
}

static void set_scale(GemmEpi& ep, const Ctx* c, const float* ss) {
  ep.ss = ss; ep.NS = (c->d / 64 + 3) & ~3; ep.eps = c->cfg.rms_eps; ep.dnorm = c->d;   // rows of ss are padded to 4 slabs
}

void mfma_gemm(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, GemmPlan p, hipStream_t s) {
  GemmEpi ep{};
  gemm_dispatch<EPI_PARTIAL>(A, W, C, M, N, K, p, ep, s);
}

// C = s_m * (A W): projection of the un-normalised bf16 residual with the RMSNorm factor applied afterwards
void mfma_gemm_scaled(Ctx* c, const bf16_t* A, const bf16_t* W, float* C, const float* ss, int M, int N, int K, GemmPlan p, hipStream_t s) {
  GemmEpi ep{};
  set_scale(ep, c, ss);
  p.splits = 1;
  gemm_dispatch<EPI_PARTIAL>(A, W, C, M, N, K, p, ep, s);
}

// x += A W; also leaves bf16(x) packed and the per-slab sums of squares of the new x
void mfma_gemm_resid(Ctx* c, const bf16_t* A, const bf16_t* W, float* x, bf16_t* xb, float* ss_out, int M, int K, hipStream_t s) {
  GemmEpi ep{};
  ep.x = x; ep.xb = xb; ep.ss_out = ss_out; ep.NS = (c->d / 64 + 3) & ~3;
  launch_gemm_direct<2, 2, 6, EPI_RESID>(A, W, nullptr, M, c->d, K, 1, ep, s);
}

// gate/up projection with the SwiGLU epilogue: act = silu(h Wg) * (h Wu), packed bf16 [M][F]
void mfma_gemm_swiglu(Ctx* c, const bf16_t* A, const bf16_t* Wgu, bf16_t* act, const float* ss, int M, int F, int K, GemmPlan p,
                      hipStream_t s) {
  GemmEpi ep{};
  set_scale(ep, c, ss);
  ep.act = act; ep.F = F;
  p.splits = 1;
  gemm_dispatch<EPI_SWIGLU>(A, Wgu, nullptr, M, 2 * F, K, p, ep, s);
}

// fused q/k/v projection with the rotary + cache-write epilogue
void mfma_gemm_qkv(Ctx* c, int layer, const bf16_t* A, const bf16_t* Wqkv, const float* ss, const TreeDesc& tree, const PosDesc& pos, int T,
                   GemmPlan p, hipStream_t s) {
  GemmEpi ep{};
  set_scale(ep, c, ss);
  ep.q = (bf16_t*)(c->ws + c->w.q);
  ep.kc = (bf16_t*)c->kv + c->kv_layer_stride * layer;
  ep.vc = (bf16_t*)c->kv + c->kv_v_off + c->kv_layer_stride * layer;
  ep.rope = (const float*)(c->ws + c->w.rope_tab);
  ep.T = T; ep.d = c->d; ep.dh = c->dh; ep.S_cap = c->S_cap; ep.rope_pos = c->rope_pos;
  ep.row_stride = c->kv_row_stride; ep.head_stride = c->kv_head_stride;
  ep.pos = pos; ep.tree = tree;
  p.splits = 1;
  gemm_dispatch<EPI_QKV>(A, Wqkv, nullptr, c->R * T, 3 * c->d, c->d, p, ep, s);
}

// ------------------------------------------------------------------------------------------------ attention
// One workgroup per (head, row).  Scores are computed transposed, S^T[key][query] = K * Q^T, so the
// accumulator layout (lane = query, registers = keys) is directly the B operand of
// O^T[dim][query] = V^T[dim][key] * P^T[key][query] and the online-softmax state of a query lives in
// one lane.  K rows ([slot][dim], dim contiguous) and V blocks ([dim][32 slots], slot contiguous) are
// loaded straight from the cache into MFMA operand registers - every key is used by exactly one wave,
// so there is nothing to share through LDS; the 4 waves take 32-key steps round-robin and merge their
// partial (max, sum, O) through LDS at the end.  Only the last T keys (the block itself) are masked.
template <int DH, int NQB, int NW>
__global__ __launch_bounds__(NW * 64) void k_attn_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc,
                                                   const bf16_t* __restrict__ vc, bf16_t* __restrict__ out, TreeDesc tree,
                                                   PosDesc pos, int T, int d, size_t row_stride, size_t head_stride, float c_exp) {
  constexpr int KD = DH / 32, DT = DH / 16, NQ = NQB * 16;
  __shared__ float s_m[NW - 1][NQ], s_l[NW - 1][NQ];
  __shared__ float s_o[NW - 1][NQ][DH + 1];
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

  // K rows / V block of one 32-key step, straight into MFMA operand registers.  S^T tile t, row i holds
  // key 8*(i/4) + 4*t + i%4 of the step, so that a lane's 8 score values are 8 consecutive keys.
#define VVS_ATTN_LOAD(STEP, KF, VF)                                                                                   \
  {                                                                                                                   \
    _Pragma("unroll") for (int t = 0; t < 2; ++t) {                                                                   \
      const int key = ((STEP) << 5) + 8 * (ql >> 2) + 4 * t + (ql & 3);                                               \
      _Pragma("unroll") for (int kd = 0; kd < KD; ++kd)                                                               \
          KF[t][kd] = as_bf16x8(*(const uint4*)(kb + (size_t)key * DH + kd * 32 + g * 8));                            \
    }                                                                                                                 \
    _Pragma("unroll") for (int dt = 0; dt < DT; ++dt)                                                                 \
        VF[dt] = as_bf16x8(*(const uint4*)(vb + ((size_t)(STEP) * DH + dt * 16 + ql) * 32 + g * 8));                  \
  }
  bf16x8 kf[2][KD], vf[DT], kn[2][KD], vn[DT];
  VVS_ATTN_LOAD(min(wave, nsteps - 1), kf, vf);
  for (int step = wave; step < nsteps; step += NW) {
    const int key0 = step << 5;
    // next step's operands are requested before this step's are used (the last iteration re-requests its own)
    VVS_ATTN_LOAD(step + NW < nsteps ? step + NW : step, kn, vn);
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
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int kd = 0; kd < KD; ++kd) kf[t][kd] = kn[t][kd];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vf[dt] = vn[dt];
  }
#undef VVS_ATTN_LOAD

  // merge the waves' partial results (waves 1.. publish, wave 0 combines and writes)
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
      for (int w = 0; w < NW - 1; ++w) m = fmaxf(m, s_m[w][qi]);
      const float m_safe = m == -INFINITY ? 0.f : m;
      const float a0 = exp2f((m_run[qb] - m_safe) * c_exp);
      float l = l_run[qb] * a0;
      float aw[NW - 1];
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) {
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
            for (int w = 0; w < NW - 1; ++w) {
              v0 += s_o[w][qi][dt * 16 + 4 * g + rr] * aw[w];
              v1 += s_o[w][qi][dt * 16 + 4 * g + rr + 1] * aw[w];
            }
            pk[rr >> 1] = (uint32_t)f2bf(v0 * inv) | ((uint32_t)f2bf(v1 * inv) << 16);
          }
          *(uint2*)(out + pack_index(r * T + qi, hd * DH + dt * 16 + 4 * g, d)) = make_uint2(pk[0], pk[1]);   // O-projection operand layout
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
#define VVS_ATTN(DH, NQB, NW)                                                                                                  \
  hipLaunchKernelGGL((k_attn_mfma<DH, NQB, NW>), grid, dim3(NW * 64), 0, s, q, kc, vc, out, tree, pos, T, c->d, c->kv_row_stride, \
                     c->kv_head_stride, c_exp)
  // 4 waves per workgroup keep the register footprint low enough for 2-3 workgroups per CU, so that
  // every (head, row) pair of a call is resident at once
  if (c->dh == 64) {
    if (nqb == 1) VVS_ATTN(64, 1, 4); else if (nqb == 2) VVS_ATTN(64, 2, 4); else VVS_ATTN(64, 4, 4);
  } else {
    if (nqb == 1) VVS_ATTN(128, 1, 4); else VVS_ATTN(128, 2, 4);   // T <= 32 is enforced at context creation for head size 128
  }
#undef VVS_ATTN
}

}  // namespace vvs
