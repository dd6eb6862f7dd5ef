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
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes as a native vector (plain register moves)

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Maximum / sum over the four lanes l % 16 + 16 j of a wave (the four 16-lane rows), left in all four, with gfx950's row
// swaps: v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second, v_permlane32_swap
// the upper half of the first with the lower half of the second - given the same value twice they return (x of the
// even / lower partner, x of the odd / upper partner) in every lane.  Plain VALU instructions: the LDS crossbar that a
// __shfl_xor goes through costs a round trip per step of these dependent chains.  Same order of additions as
// x += xor16(x); x += xor32(x).
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float rows_max(float x) {
  uintx2 p = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(p[0]), __uint_as_float(p[1]));
  p = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(p[0]), __uint_as_float(p[1]));
}
__device__ __forceinline__ float rows_sum(float x) {
  uintx2 p = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(p[0]) + __uint_as_float(p[1]);
  p = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(p[0]) + __uint_as_float(p[1]);
}

// Phase marks: a profiling build may define VVS_PHASE_MARK(i) to record a time stamp at the i-th
// point of a kernel (entry, operands requested, main loop done, tile in LDS, end); normally nothing.
#ifndef VVS_PHASE_MARK
#define VVS_PHASE_MARK(i)
#endif

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
//                thread), also written, times the gain of the norm that follows, as the packed bf16
//                operand of the next projection, plus the sum of squares of the tile's 64 columns per
//                row (one K split only).
// Row scale: RMSNorm is x * s_m * g with s_m = rsqrt(mean_k x_mk^2 + eps).  The operand of the projection
// behind a norm is bf16(x * g), written by whoever produced x, and s_m - a per-row factor that commutes
// with the contraction - multiplies the accumulated tile in the epilogue; s_m comes from the
// per-64-column sums of squares that the producer of x (EPI_RESID or the embedding kernel) left in ss.
// This removes the separate normalisation pass between two projections; the weights stay as given.
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_QKV = 2, EPI_RESID = 3 };

struct GemmEpi {
  const float* ss; int NS; float eps; int dnorm;           // row scale (ss == nullptr: no scaling); ss[M][NS]
  bf16_t* act; int F;                                      // EPI_SWIGLU
  float* x; bf16_t* xb; float* ss_out; const float* g_next; // EPI_RESID (g_next: gain of the norm that reads x next)
  int xb_T, xb_pad;                                        // EPI_RESID: xb_T > 0 = xb in the row-padded layout (row m at (m / xb_T) * xb_pad + m % xb_T)
  bf16_t* q; bf16_t* kc; bf16_t* vc; const float* rope;    // EPI_QKV
  int T, d, dh, S_cap, rope_pos;
  int row_owner;                                           // tile order of the direct-to-LDS kernel: 1 = an XCD owns row tiles
  size_t row_stride, head_stride;
  PosDesc pos;
  TreeDesc tree;
};

// Per-row RMSNorm factor of a tile's rows, from the per-slab sums of squares (1 when the GEMM is not
// scaled), in two phases: the loads are issued when the kernel starts and their values are only used
// after the main loop, so their latency is never waited for.  4 lanes per row (unit = row * 4 + part),
// each takes every 4th group of 4 slabs; RU = BM * 4 / 256 units per thread.
template <int BM>
struct RowScale {
  static constexpr int RU = (BM * 4 + 255) / 256;
  float4 v[RU][4];
  __device__ __forceinline__ void load(int tile_m, int M, const GemmEpi& ep) {
#pragma unroll
    for (int j = 0; j < RU; ++j) {
      const int u = threadIdx.x + 256 * j, row = u >> 2, part = u & 3;
      const int m = min(tile_m * BM + row, M - 1);                       // clamped rows are never stored
      const int nq = ep.NS >> 2;                                         // rows of ss are padded to a multiple of 4 slabs (zeros)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        v[j][i] = (ep.ss && part + 4 * i < nq) ? ((const float4*)(ep.ss + (size_t)m * ep.NS))[part + 4 * i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  __device__ __forceinline__ void finish(float* rs, int tile_m, int M, const GemmEpi& ep) {
#pragma unroll
    for (int j = 0; j < RU; ++j) {
      const int u = threadIdx.x + 256 * j, row = u >> 2, part = u & 3;
      const int m = min(tile_m * BM + row, M - 1);
      float t = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) t += (v[j][i].x + v[j][i].y) + (v[j][i].z + v[j][i].w);
      if (ep.ss)
        for (int qd = part + 16; qd < (ep.NS >> 2); qd += 4) {           // more than 64 slabs: the rest is read here
          const float4 w = ((const float4*)(ep.ss + (size_t)m * ep.NS))[qd];
          t += (w.x + w.y) + (w.z + w.w);
        }
      t += __shfl_xor(t, 1, 64);
      t += __shfl_xor(t, 2, 64);
      if (part == 0 && row < BM) rs[row] = ep.ss ? 1.0f / sqrtf(t / (float)ep.dnorm + ep.eps) : 1.f;
    }
  }
};

// Epilogue inputs that do not depend on the accumulators are requested early, so that their latency
// hides behind the main loop instead of being paid after it.
//   EPI_RESID: the residual values the tile will be added to (requested behind the first operand loads).
//   EPI_QKV  : a thread owns tile row tid % BM.  first() requests the cache length / emitted count
//              behind that row's position before any operand load (loads return in order, so these
//              come back first); after the first operand loads are on their way, rope() turns them
//              into (slot, image index) and requests this thread's share of the row's rotary factors -
//              contiguous 16-byte pieces of the table rows of the token's grid row and column;
//              to_lds() leaves slot, image index and factors in LDS for the epilogue, which so reads
//              them with a few wide LDS loads instead of 16 scattered global loads per unit.
constexpr int kRopeNpMax = 16;   // rotary pairs per position kept in LDS (head size 64); other head sizes read the table directly
template <int BM, int BN, int EPI, bool EARLY = true>
struct EpiPre {
  // EARLY = false (large tiles, where the early copies would not fit the register file): EPI_RESID reads the residual
  // and the gain in the epilogue itself
  static constexpr int UR = (BM * (BN / 8) + 255) / 256;    // EPI_RESID units (row, 8 columns) per thread
  static constexpr int URE = EARLY ? UR : 1;
  static constexpr int G = 256 / BM;                        // threads per tile row
  static constexpr int NR = 2 * kRopeNpMax / G / 2;         // float4 (two factor pairs) per thread
  int kv, ne, slot, img;
  bool rope_lds = true;          // false: the epilogue reads the rotary table from memory (kernels that keep no per-row table in LDS)
  float4 rp[NR];
  float4 x0[URE], x1[URE], g0[URE], g1[URE];

  // m / T for 0 <= m < 2^20 (the quotient of the rounded product cannot cross an integer: the exact
  // value is at least 0.5 / T away from one)
  __device__ __forceinline__ static int div_T(int m, const GemmEpi& ep) { return (int)(((float)m + 0.5f) * (1.0f / (float)ep.T)); }

  __device__ __forceinline__ void first(int tile_m, int M, const GemmEpi& ep) {
    if constexpr (EPI == EPI_QKV) {
      kv = ne = 0;
      if (ep.pos.kv_len) {
        const int b = div_T(min(tile_m * BM + (int)threadIdx.x % BM, M - 1), ep) >> 1;
        kv = ep.pos.kv_len[b];
        ne = ep.pos.n_emitted[b];
      }
    }
  }
  __device__ __forceinline__ void start(int tile_m, int tile_n, int M, int N, const GemmEpi& ep) {
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    if constexpr (EPI == EPI_QKV) {
      const int m = min(m0 + (int)threadIdx.x % BM, M - 1), t = m - div_T(m, ep) * ep.T;
      if (ep.pos.kv_len) {
        slot = kv + t;
        img = ne - 1 + ep.tree.depth[t];
      } else {
        slot = ep.pos.kv_base + t;
        img = slot - ep.pos.prefix_len;
      }
      const int np = ep.dh >> 2;
      if (n0 / ep.d < 2 && np == kRopeNpMax && rope_lds) {   // q and k columns are rotated
        const int im = max(img, 0), gr = min(im / ep.pos.grid_w, ep.rope_pos - 1), gc = im % ep.pos.grid_w;
        // the row's 2 * np pairs, [grid row: np][grid column: np], are dealt to its G threads in order
        const int per = 2 * np / G, p0 = ((int)threadIdx.x / BM) * per;   // pairs per thread (even), first pair
#pragma unroll
        for (int i = 0; i < NR; ++i) {
          const int pr = min(p0 + 2 * i, 2 * np - 2), pv = pr >= np ? gc : gr, ip = pr >= np ? pr - np : pr;
          rp[i] = *(const float4*)(ep.rope + ((size_t)pv * np + ip) * 2);
        }
      }
    } else if constexpr (EPI == EPI_RESID && EARLY) {
#pragma unroll
      for (int j = 0; j < UR; ++j) {
        const int u = threadIdx.x + 256 * j, row = min(u / (BN / 8), BM - 1), c8 = (u % (BN / 8)) * 8;
        const float* xp = ep.x + (size_t)min(m0 + row, M - 1) * N + n0 + c8;   // clamped rows are never stored
        x0[j] = *(const float4*)xp;
        x1[j] = *(const float4*)(xp + 4);
        g0[j] = *(const float4*)(ep.g_next + n0 + c8);
        g1[j] = *(const float4*)(ep.g_next + n0 + c8 + 4);
      }
    }
  }
  // s_pos[BM][2] = (slot, image index); s_rope[BM][2 * kRopeNpMax] = (cos, sin) pairs, grid-row half then grid-column half
  __device__ __forceinline__ void to_lds(int* s_pos, float2* s_rope, const GemmEpi& ep) const {
    if constexpr (EPI == EPI_QKV) {
      const int row = threadIdx.x % BM, g = threadIdx.x / BM, np = ep.dh >> 2;
      if (g == 0) { s_pos[2 * row] = slot; s_pos[2 * row + 1] = img; }
      if (np == kRopeNpMax && rope_lds) {
        const int per = 2 * np / G, p0 = g * per;
#pragma unroll
        for (int i = 0; i < NR; ++i)
          if (2 * i < per) *(float4*)(s_rope + row * 2 * kRopeNpMax + p0 + 2 * i) = rp[i];
      }
    }
  }
};

// Epilogue of a BM x BN tile whose NP partial sums lie in LDS as red[NP][BM][BN + 4] (added in a fixed
// order); rs holds the row factors.  Called by all 256 threads after a barrier.
template <int BM, int BN, int NP, int EPI, bool EARLY = true>
__device__ __forceinline__ void tile_epilogue(const float* red, const float* rs, int tile_m, int tile_n, int M, int N, float* C,
                                              const GemmEpi& ep, const EpiPre<BM, BN, EPI, EARLY>& pre, const int* s_pos, const float2* s_rope) {
  constexpr int LDC = BN + 4;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  constexpr int PS = BM * LDC;   // stride between the partial tiles
  // sum of the partial tiles for 4 consecutive columns, fixed order
  auto sum4 = [&](const float* p) {
    float4 a = *(const float4*)p;
#pragma unroll
    for (int w = 1; w < NP; ++w) {
      const float4 b = *(const float4*)(p + w * PS);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    return a;
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
    static_assert(BN % 64 == 0, "gate / up blocks of 32 columns alternate inside the tile");
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
        // silu(g) * up with the hardware exp2 and reciprocal (1 ulp each): the epilogue is VALU work of a single wave per SIMD
        v[i] = g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * up;
      }
      store8(ep.act, m0 + row, tile_n * (BN / 2) + fl, ep.F, v);
    }
  } else if constexpr (EPI == EPI_RESID) {
    static_assert(BN % 64 == 0, "the sums of squares are kept per 64-column slab");
#pragma unroll
    for (int j = 0; j < EpiPre<BM, BN, EPI>::UR; ++j) {            // one unit = (row, 8 consecutive columns); 8 lanes share a row and slab
      const int u = threadIdx.x + 256 * j, row = u / (BN / 8), c8 = (u % (BN / 8)) * 8;
      const int m = m0 + row;
      float sq = 0.f;
      if (row < BM && m < M) {
        const float4 a = sum4(red + row * LDC + c8), b = sum4(red + row * LDC + c8 + 4);
        float* xp = ep.x + (size_t)m * N + n0 + c8;
        float4 xa, xb4, ga, gb;
        if constexpr (EARLY) {
          xa = pre.x0[j]; xb4 = pre.x1[j]; ga = pre.g0[j]; gb = pre.g1[j];
        } else {
          xa = *(const float4*)xp; xb4 = *(const float4*)(xp + 4);
          ga = *(const float4*)(ep.g_next + n0 + c8); gb = *(const float4*)(ep.g_next + n0 + c8 + 4);
        }
        float v[8] = {xa.x + a.x, xa.y + a.y, xa.z + a.z, xa.w + a.w, xb4.x + b.x, xb4.y + b.y, xb4.z + b.z, xb4.w + b.w};
        *(float4*)xp = make_float4(v[0], v[1], v[2], v[3]);
        *(float4*)(xp + 4) = make_float4(v[4], v[5], v[6], v[7]);
        const float hv[8] = {v[0] * ga.x, v[1] * ga.y, v[2] * ga.z, v[3] * ga.w, v[4] * gb.x, v[5] * gb.y, v[6] * gb.z, v[7] * gb.w};
        store8(ep.xb, ep.xb_T > 0 ? (m / ep.xb_T) * ep.xb_pad + m % ep.xb_T : m, n0 + c8, N, hv);
#pragma unroll
        for (int i = 0; i < 8; ++i) sq += v[i] * v[i];
      }
      sq += __shfl_xor(sq, 1, 64);
      sq += __shfl_xor(sq, 2, 64);
      sq += __shfl_xor(sq, 4, 64);
      if (row < BM && m < M && (c8 & 63) == 0) ep.ss_out[(size_t)m * ep.NS + tile_n * (BN / 64) + (c8 >> 6)] = sq;
    }
  } else {
    const int sec = n0 / ep.d;                                     // the tile lies inside the q (0), k (1) or v (2) third
    // index arithmetic without per-thread integer divisions: the tile's first column inside its third is
    // uniform, and the head size of this path is a power of two (64 or 128)
    const int nd = n0 - sec * ep.d, dh_sh = 31 - __clz(ep.dh), dh_mask = ep.dh - 1;
    if (sec == 0) {
      const int half = ep.dh >> 1, np = ep.dh >> 2;
      for (int u = threadIdx.x; u < BM * (BN / 16); u += 256) {    // q: one unit = (row, 16 consecutive columns), row-major output
        const int row = u / (BN / 16), c0 = (u % (BN / 16)) * 16;
        const int m = m0 + row;
        if (m >= M) continue;
        const float* p = red + row * LDC + c0;
        const float4 s0 = sum4(p), s1 = sum4(p + 4), s2 = sum4(p + 8), s3 = sum4(p + 12);
        float v[16] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w, s2.x, s2.y, s2.z, s2.w, s3.x, s3.y, s3.z, s3.w};
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] *= rs[row];
        const int eg = nd + c0, e = eg & dh_mask;
        const int img = s_pos[2 * row + 1];
        if (img >= 0) {
          float2 cs[8];
          if (np == kRopeNpMax && s_rope) {
            // 16 columns = 8 pairs inside one half of the head: 8 consecutive pairs of the row's LDS table
            const float4* t4 = (const float4*)(s_rope + row * 2 * kRopeNpMax + (e >> (dh_sh - 1)) * np + ((e & (half - 1)) >> 1));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float4 c4 = t4[i];
              cs[2 * i] = make_float2(c4.x, c4.y);
              cs[2 * i + 1] = make_float2(c4.z, c4.w);
            }
          } else {
            const int gr = min(img / ep.pos.grid_w, ep.rope_pos - 1), gc = img % ep.pos.grid_w;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const int ei = e + 2 * i, pv = (ei >> (dh_sh - 1)) ? gc : gr, ip = (ei & (half - 1)) >> 1;
              cs[i] = *(const float2*)(ep.rope + ((size_t)pv * np + ip) * 2);
            }
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float a = v[2 * i], b = v[2 * i + 1];
            v[2 * i] = a * cs[i].x - b * cs[i].y;
            v[2 * i + 1] = a * cs[i].y + b * cs[i].x;
          }
        }
        uint4* dst = (uint4*)(ep.q + (size_t)m * ep.d + eg);
        dst[0] = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]),
                            pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
        dst[1] = make_uint4(pack2bf(v[8], v[9]), pack2bf(v[10], v[11]),
                            pack2bf(v[12], v[13]), pack2bf(v[14], v[15]));
      }
    } else if (sec == 1) {
      // k: in the cache's operand order 4 consecutive slots of one 8-dim piece are contiguous, so a lane
      // takes one row (token) and the lanes of a wave cover consecutive tokens; a thread handles
      // 8-column pieces (one 16-byte store each) of its row.
      constexpr int G = 256 / BM;                                  // threads per row
      const int half = ep.dh >> 1, np = ep.dh >> 2;
      const int row = threadIdx.x % BM, g4 = threadIdx.x / BM, m = m0 + row;
      const int slot = pre.slot, img = pre.img;                    // this thread's row is the one it looked up
      if (m < M && slot >= 0 && slot < ep.S_cap) {
        const float sc = rs[row];
        bf16_t* krow = ep.kc + (size_t)EpiPre<BM, BN, EPI>::div_T(m, ep) * ep.row_stride;
        const int gr = min(max(img, 0) / ep.pos.grid_w, ep.rope_pos - 1), gc = max(img, 0) % ep.pos.grid_w;
#pragma unroll 2
        for (int c8 = g4 * 8; c8 < BN; c8 += G * 8) {
          const float4 a = sum4(red + row * LDC + c8), b = sum4(red + row * LDC + c8 + 4);
          float v[8] = {a.x * sc, a.y * sc, a.z * sc, a.w * sc, b.x * sc, b.y * sc, b.z * sc, b.w * sc};
          const int eg = nd + c8, hd = eg >> dh_sh, e = eg & dh_mask;
          if (img >= 0) {
            float2 cs[4];
            if (np == kRopeNpMax && s_rope) {
              const float4* t4 = (const float4*)(s_rope + row * 2 * kRopeNpMax + (e >> (dh_sh - 1)) * np + ((e & (half - 1)) >> 1));
              const float4 c0 = t4[0], c1 = t4[1];
              cs[0] = make_float2(c0.x, c0.y); cs[1] = make_float2(c0.z, c0.w);
              cs[2] = make_float2(c1.x, c1.y); cs[3] = make_float2(c1.z, c1.w);
            } else {
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const int ei = e + 2 * i, pv = (ei >> (dh_sh - 1)) ? gc : gr, ip = (ei & (half - 1)) >> 1;
                cs[i] = *(const float2*)(ep.rope + ((size_t)pv * np + ip) * 2);
              }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float x0 = v[2 * i], x1 = v[2 * i + 1];
              v[2 * i] = x0 * cs[i].x - x1 * cs[i].y;
              v[2 * i + 1] = x0 * cs[i].y + x1 * cs[i].x;
            }
          }
          *(uint4*)(krow + (size_t)hd * ep.head_stride + k_index(slot, e, ep.dh)) =
              make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]),
                         pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
        }
      }
    } else {
      // v: the cache keeps the 32 slots of a dim contiguous, so a lane takes one row (token) and the lanes of
      // a wave cover consecutive tokens: one store instruction then writes runs of consecutive slots of one
      // dim instead of 64 different lines.  A thread reads 4 consecutive columns (float4) of its row.
      constexpr int G = 256 / BM;                                  // threads per row
      const int row = threadIdx.x % BM, g = threadIdx.x / BM, m = m0 + row;
      const int slot = pre.slot;                                   // this thread's row is the one it looked up
      if (m < M && slot >= 0 && slot < ep.S_cap) {
        const float sc = rs[row];
        bf16_t* vrow = ep.vc + (size_t)EpiPre<BM, BN, EPI>::div_T(m, ep) * ep.row_stride;
#pragma unroll 4
        for (int c4 = g * 4; c4 < BN; c4 += G * 4) {
          const float4 v = sum4(red + row * LDC + c4);
          const int eg = nd + c4, hd = eg >> dh_sh, e = eg & dh_mask;    // 4 columns stay inside one head
          bf16_t* vh = vrow + (size_t)hd * ep.head_stride;
          vh[v_index(slot, e, ep.dh)] = f2bf(v.x * sc);
          vh[v_index(slot, e + 1, ep.dh)] = f2bf(v.y * sc);
          vh[v_index(slot, e + 2, ep.dh)] = f2bf(v.z * sc);
          vh[v_index(slot, e + 3, ep.dh)] = f2bf(v.w * sc);
        }
      }
    }
  }
}


template <int TM, int TN, int D, int EPI>
__global__ __launch_bounds__(256) void k_gemm_direct(const uint4* __restrict__ Ap, const uint4* __restrict__ Wp, float* __restrict__ C,
                                                     int M, int N, int K, int kb_per_split, const GemmEpi ep) {
  constexpr int BM = TM * 32, BN = TN * 32, LDC = BN + 4;
  extern __shared__ float red[];           // [4][BM][LDC]
  VVS_PHASE_MARK(0);
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
  __shared__ float rs[BM];                 // per-row RMSNorm factor of this tile's rows
  __shared__ int s_pos[EPI == EPI_QKV ? 2 * BM : 2];                                  // EPI_QKV: (slot, image index) per tile row
  __shared__ __align__(16) float2 s_rope[EPI == EPI_QKV ? BM * 2 * kRopeNpMax : 2];   // EPI_QKV: rotary factors per tile row
  EpiPre<BM, BN, EPI> pre;
  pre.first(tile_m, M, ep);
  __builtin_amdgcn_sched_barrier(0);
  const int KB = K >> 4;
  const int s0 = blockIdx.z * kb_per_split, s1 = min(KB, s0 + kb_per_split);
  const int per_w = (max(s1 - s0, 0) + 3) >> 2;
  const int w0 = s0 + wave * per_w, w1 = min(s1, w0 + per_w);
  const int nk = max(w1 - w0, 0);
  const uint4* ap[TM];
  const uint4* bp[TN];
#pragma unroll
  for (int t = 0; t < TM; ++t) ap[t] = Ap + ((size_t)min(tile_m * TM + t, (M - 1) >> 5) * KB) * 64 + lane;   // row blocks past the end repeat the last one
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
  // epilogue inputs: requested behind the first operand loads (nothing waits for them before the main loop ends)
  RowScale<BM> rowscale;
  rowscale.load(tile_m, M, ep);
  if (EPI != EPI_QKV || nk <= 0) pre.start(tile_m, tile_n, M, N, ep);
  __builtin_amdgcn_sched_barrier(0);
  VVS_PHASE_MARK(1);
  for (int kb = 0; kb < nk; kb += D) {
    // EPI_QKV: the rotary factors depend on a loaded value (the row's cache length); asking for them after the
    // first group of k-steps instead of in front of the loop keeps that wait off the path to the first MFMA
    if (EPI == EPI_QKV && kb == D) pre.start(tile_m, tile_n, M, N, ep);
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
  if (EPI == EPI_QKV && nk > 0 && nk <= D) pre.start(tile_m, tile_n, M, N, ep);   // a K range of a single group
  VVS_PHASE_MARK(2);
  pre.to_lds(s_pos, s_rope, ep);
  rowscale.finish(rs, tile_m, M, ep);
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
  VVS_PHASE_MARK(3);
  tile_epilogue<BM, BN, 4, EPI>(red, rs, tile_m, tile_n, M, N, C, ep, pre, s_pos, s_rope);
  VVS_PHASE_MARK(4);
}

// Shared-operand variant for projections with enough output tiles: a workgroup owns a
// (2*WM*32) x (2*WN*32) tile, its 4 waves form a 2 x 2 grid of (WM*32) x (WN*32) sub-tiles and all of
// them read the A and B fragments from LDS, so every operand byte that comes through the CU's L1 feeds
// twice as many MFMAs as in k_gemm_direct.  A stage is 32 contraction indices = 2 fragment blocks per
// 32 rows; the blocks are copied global -> registers -> LDS as they are (the packed layout is already
// the LDS layout the MFMA lanes want).
// Software pipeline (one wave per SIMD, so nothing else hides latencies): global loads run D stages
// ahead in registers; LDS holds 3 stages; in iteration s a wave requests the second half of stage s from
// LDS, moves stage s+2 from registers to LDS and re-requests those registers from memory, multiplies
// the first half of stage s, requests the first half of stage s+1 and multiplies the second half:
// every MFMA group runs on fragments requested one group earlier.  One barrier per stage: it orders
// the LDS writes of stage s+2 before their reads in iteration s+1 and the reads of stage s before the
// slot is overwritten in iteration s+1.  The epilogues are the same as above with a single partial tile.
template <int WM, int WN, int D, int EPI>
__global__ __launch_bounds__(256) void k_gemm_shared(const uint4* __restrict__ Ap, const uint4* __restrict__ Wp, float* __restrict__ C,
                                                     int M, int N, int K, const GemmEpi ep) {
  constexpr int BM = 2 * WM * 32, BN = 2 * WN * 32, LDC = BN + 4;
  constexpr int NA = 2 * (BM / 32), NBLK = NA + 2 * (BN / 32), PER = NBLK / 4;   // 1 KiB blocks per stage; per wave
  static_assert(NBLK % 4 == 0, "blocks of a stage are dealt to 4 waves");
  static_assert(D % 3 == 0, "register ring and LDS ring indices are both static after unrolling by D");
  extern __shared__ float red[];           // main loop: u32x4 stage[3][NBLK][64]; afterwards: float [BM][LDC]
  u32x4* stage = (u32x4*)red;
  VVS_PHASE_MARK(0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int MT = (M + BM - 1) / BM, NT = N / BN;
  int tile_m, tile_n;
  {                                        // same XCD-aware order as k_gemm_direct
    const int id = blockIdx.x, grp = id / (8 * MT), rem = id % (8 * MT);
    const int cols = min(8, NT - grp * 8);
    tile_m = rem / cols;
    tile_n = grp * 8 + rem % cols;
  }
  __shared__ float rs[BM];
  __shared__ int s_pos[EPI == EPI_QKV ? 2 * BM : 2];                                  // EPI_QKV: (slot, image index) per tile row
  __shared__ __align__(16) float2 s_rope[EPI == EPI_QKV ? BM * 2 * kRopeNpMax : 2];   // EPI_QKV: rotary factors per tile row
  EpiPre<BM, BN, EPI> pre;
  pre.first(tile_m, M, ep);
  __builtin_amdgcn_sched_barrier(0);
  const int KB = K >> 4, nst = KB >> 1;
  const int last_rb = (M - 1) >> 5;        // row blocks past the end of A repeat the last one (their rows are never stored)
  // block j of a stage: j < NA: A row block j/2, else B row block (j-NA)/2; contraction block 2*s + j%2
  const u32x4* src[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int j = wave + 4 * i;
    const int rb = j < NA ? min(tile_m * (BM / 32) + (j >> 1), last_rb) : tile_n * (BN / 32) + ((j - NA) >> 1);
    src[i] = (const u32x4*)(j < NA ? Ap : Wp) + ((size_t)rb * KB + (j & 1)) * 64 + lane;
  }
  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  // stage t lives in st[t % D] until it is written to LDS slot t % 3; stages past the end repeat the last one
  u32x4 st[D][PER];
#define VVS_G2R(RD, T)                                                                                                \
  {                                                                                                                   \
    const size_t kk = (size_t)min((T), nst - 1) * 128;                                                                \
    _Pragma("unroll") for (int i = 0; i < PER; ++i) st[RD][i] = src[i][kk];                                           \
    __builtin_amdgcn_sched_barrier(0); /* load groups stay in program order: waits are partial */                     \
  }
#define VVS_R2S(RD, SL) \
  { _Pragma("unroll") for (int i = 0; i < PER; ++i) stage[((SL) * NBLK + wave + 4 * i) * 64 + lane] = st[RD][i]; }
#define VVS_S2F(FA, FB, SL, KBO)                                                                                      \
  {                                                                                                                   \
    _Pragma("unroll") for (int t = 0; t < WM; ++t)                                                                    \
        FA[t] = __builtin_bit_cast(bf16x8, stage[((SL) * NBLK + (wr * WM + t) * 2 + (KBO)) * 64 + lane]);             \
    _Pragma("unroll") for (int t = 0; t < WN; ++t)                                                                    \
        FB[t] = __builtin_bit_cast(bf16x8, stage[((SL) * NBLK + NA + (wc * WN + t) * 2 + (KBO)) * 64 + lane]);        \
  }
#define VVS_MMA(FA, FB)                                                                                               \
  {                                                                                                                   \
    _Pragma("unroll") for (int ti = 0; ti < WM; ++ti)                                                                 \
        _Pragma("unroll") for (int tj = 0; tj < WN; ++tj)                                                             \
            acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[ti], FB[tj], acc[ti][tj], 0, 0, 0);              \
  }
#pragma unroll
  for (int d = 0; d < D; ++d) VVS_G2R(d, d)
  // epilogue inputs: requested behind the first operand loads (nothing waits for them before the main loop ends)
  RowScale<BM> rowscale;
  rowscale.load(tile_m, M, ep);
  pre.start(tile_m, tile_n, M, N, ep);
  __builtin_amdgcn_sched_barrier(0);
  VVS_PHASE_MARK(1);
  VVS_R2S(0, 0)
  VVS_G2R(0, D)
  VVS_R2S(1, 1)
  VVS_G2R(1, D + 1)
  __syncthreads();
  bf16x8 fa0[WM], fb0[WN], fa1[WM], fb1[WN];
  VVS_S2F(fa0, fb0, 0, 0)
  // iteration S with d = S % D (so S % 3 == d % 3)
#define VVS_ITER(S)                                                                                                   \
  {                                                                                                                   \
    VVS_S2F(fa1, fb1, d % 3, 1)                                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                                                \
    VVS_R2S((d + 2) % D, (d + 2) % 3)                                                                                 \
    VVS_G2R((d + 2) % D, (S) + 2 + D)                                                                                 \
    VVS_MMA(fa0, fb0)                                                                                                 \
    __builtin_amdgcn_sched_barrier(0);                                                                                \
    VVS_S2F(fa0, fb0, (d + 1) % 3, 0)                                                                                 \
    __builtin_amdgcn_sched_barrier(0);                                                                                \
    VVS_MMA(fa1, fb1)                                                                                                 \
    __syncthreads();                                                                                                  \
  }
  // whole groups of D iterations run without any condition, so that the wait before a stage's LDS
  // write is "all but the D-1 younger load groups"
  int s0 = 0;
  for (; s0 + D <= nst; s0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) VVS_ITER(s0 + d)
  }
#pragma unroll
  for (int d = 0; d < D; ++d)
    if (s0 + d < nst) VVS_ITER(s0 + d)                         // uniform over the workgroup
#undef VVS_ITER
#undef VVS_MMA
#undef VVS_S2F
#undef VVS_R2S
#undef VVS_G2R
  VVS_PHASE_MARK(2);
  pre.to_lds(s_pos, s_rope, ep);
  rowscale.finish(rs, tile_m, M, ep);
  __syncthreads();                         // the stage buffers become the output tile
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        red[((wr * WM + i) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * LDC + (wc * WN + j) * 32 + (lane & 31)] = acc[i][j][r];
  __syncthreads();
  VVS_PHASE_MARK(3);
  tile_epilogue<BM, BN, 1, EPI>(red, rs, tile_m, tile_n, M, N, C, ep, pre, s_pos, s_rope);
  VVS_PHASE_MARK(4);
}

// The same tile with the stages loaded straight from global memory into LDS (global_load_lds_dwordx4: lane l
// of a wave writes the 16 bytes it asked for to LDS address M0 + 16 l, which is exactly the packed block
// layout).  In k_gemm_shared every operand byte crosses the vector registers twice - once on its way from
// memory to LDS, once as a fragment - and the register file's ports, shared with the MFMA operand reads, are
// what that kernel's main loop is bound by; here the staging hop is gone, and so are its registers, so NS = 8
// stages can be in flight in LDS.  The compiler knows nothing of these loads (inline asm): the waits are
// written out by hand.  Iteration s: request stage s + NS - 1 into the slot stage s - 1 has left; multiply
// (fragments as in k_gemm_shared); wait until this wave's part of stage s + 2 has landed - loads return in
// order, so "at most PER * (NS - 3) younger loads outstanding" - and meet the other waves at the barrier.
// M0 is written here, so it is on the clobber list: the compiler must not keep a value of its own in it across
// the statement (it names M0 "reserved" and warns about any clobber of it; that warning is silenced for this
// one statement).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_dma16(const void* g, uint32_t lds_byte_addr) {
  const uint32_t a = __builtin_amdgcn_readfirstlane(lds_byte_addr);     // wave-uniform by construction
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(a), "v"(g) : "memory", "m0");
}
#pragma clang diagnostic pop
// L1 fill probe (vvs_debug_fill_probe): every workgroup reads the same region `reps` times; a wave takes 1 KiB blocks
// round-robin, 8 in flight.  DMA: the blocks go straight to LDS (8 slots per wave), else into registers.
template <bool DMA>
__global__ __launch_bounds__(1024) void k_fill_probe(const uint4* __restrict__ src0, size_t wg_stride16, int n_blocks, int reps,
                                                     uint32_t* __restrict__ sink) {
  extern __shared__ float probe_lds[];     // DMA: 8 KiB per wave
  const uint4* src = src0 + (size_t)blockIdx.x * wg_stride16;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const uint32_t slot0 = (uint32_t)(uintptr_t)probe_lds + (uint32_t)wave * 8192u;
  uint32_t acc = 0;
  for (int rep = 0; rep < reps; ++rep) {
    for (int blk = wave; blk < n_blocks; blk += nw * 8) {
      if constexpr (DMA) {
#pragma unroll
        for (int u = 0; u < 8; ++u) lds_dma16(src + (size_t)min(blk + u * nw, n_blocks - 1) * 64 + lane, slot0 + (uint32_t)u * 1024u);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the slots are reused by the next round
      } else {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(size_t)min(blk + u * nw, n_blocks - 1) * 64 + lane];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (v[u].x ^ v[u].y) ^ (v[u].z ^ v[u].w);   // all four words: the loads stay 16 bytes wide
      }
    }
  }
  asm volatile("" ::"v"(acc));
  if (threadIdx.x == 0) sink[blockIdx.x] = acc;
}

void launch_fill_probe(const void* src, size_t region_bytes, size_t wg_stride_bytes, int reps, int mode, int n_workgroups, int waves,
                       uint32_t* sink, hipStream_t s) {
  const int n_blocks = (int)(region_bytes >> 10);
  if (mode == 1) {
    const size_t lds = (size_t)waves * 8192;
    allow_dynamic_lds(reinterpret_cast<const void*>(&k_fill_probe<true>), lds);
    hipLaunchKernelGGL(k_fill_probe<true>, dim3(n_workgroups), dim3(waves * 64), lds, s, (const uint4*)src, wg_stride_bytes >> 4, n_blocks, reps, sink);
  } else {
    hipLaunchKernelGGL(k_fill_probe<false>, dim3(n_workgroups), dim3(waves * 64), 0, s, (const uint4*)src, wg_stride_bytes >> 4, n_blocks, reps, sink);
  }
}

template <int WM, int WN, int NS, int EPI>
__global__ __launch_bounds__(256) void k_gemm_shared_dma(const uint4* __restrict__ Ap, const uint4* __restrict__ Wp, float* __restrict__ C,
                                                         int M, int N, int K, const GemmEpi ep) {
  static_assert(NS >= 4, "at least three stages in flight");
  constexpr int BM = 2 * WM * 32, BN = 2 * WN * 32, LDC = BN + 4;
  // The output tile goes through LDS for the epilogue.  A tile too large for that (256 x 256) goes in RP = 2 passes of
  // BM / 2 rows - the rows of one wave row - so that LDS only ever holds half of it.
  constexpr int RP = (size_t)BM * LDC * sizeof(float) > 140 * 1024 ? 2 : 1, EM = BM / RP;
  constexpr int NA = 2 * (BM / 32), NBLK = NA + 2 * (BN / 32), PER = NBLK / 4;
  static_assert(NBLK % 4 == 0, "blocks of a stage are dealt to 4 waves");
  static_assert(PER * (NS - 1) <= 60, "the load counter has 6 bits");
  extern __shared__ float red[];           // main loop: u32x4 stage[NS][NBLK][64]; afterwards: float [BM][LDC]
  u32x4* stage = (u32x4*)red;
  const uint32_t lds_base = (uint32_t)(uintptr_t)stage;
  VVS_PHASE_MARK(0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int MT = (M + BM - 1) / BM, NT = N / BN;
  int tile_m, tile_n;
  if (!ep.row_owner) {                     // same XCD-aware order as k_gemm_direct: an XCD owns column tiles (weights fetched once,
    const int id = blockIdx.x, grp = id / (8 * MT), rem = id % (8 * MT);   // the activation operand once per XCD)
    const int cols = min(8, NT - grp * 8);
    tile_m = rem / cols;
    tile_n = grp * 8 + rem % cols;
  } else {                                 // the transposed order: an XCD owns row tiles (activations fetched once, the weights once
    const int id = blockIdx.x, grp = id / (8 * NT), rem = id % (8 * NT);   // per XCD): for many rows and few columns the
    const int rows = min(8, MT - grp * 8);                                 // activation operand is the larger one
    tile_n = rem / rows;
    tile_m = grp * 8 + rem % rows;
  }
  __shared__ float rs[BM];
  __shared__ int s_pos[EPI == EPI_QKV ? 2 * BM : 2];    // EPI_QKV: (slot, image index) per tile row; the rotary factors are read from
                                                        // their table in memory (an LDS copy per row would keep a second workgroup off the CU)
  constexpr bool EARLY = EPI != EPI_RESID;   // the residual tile is read in the epilogue: early copies of a tile this size do not fit the registers
  EpiPre<EM, BN, EPI, EARLY> pre[RP];        // epilogue inputs of each pass (a pass is a tile of EM rows at row tile tile_m * RP + p)
#pragma unroll
  for (int p = 0; p < RP; ++p) pre[p].rope_lds = false;
  const int KB = K >> 4, nst = KB >> 1;
  const int last_rb = (M - 1) >> 5;
  RowScale<BM> rowscale;                   // the epilogue's inputs first: they are the oldest loads and so never wait behind a stage
#pragma unroll
  for (int p = 0; p < RP; ++p) pre[p].first(tile_m * RP + p, M, ep);
  rowscale.load(tile_m, M, ep);
  if (EPI != EPI_QKV) {
#pragma unroll
    for (int p = 0; p < RP; ++p) pre[p].start(tile_m * RP + p, tile_n, M, N, ep);
  }
  __builtin_amdgcn_sched_barrier(0);
  const u32x4* src[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int j = wave + 4 * i;
    const int rb = j < NA ? min(tile_m * (BM / 32) + (j >> 1), last_rb) : tile_n * (BN / 32) + ((j - NA) >> 1);
    src[i] = (const u32x4*)(j < NA ? Ap : Wp) + ((size_t)rb * KB + (j & 1)) * 64 + lane;
  }
  // stage t -> slot t % NS; stages past the end repeat the last one (never read)
  auto request = [&](int t) {
    const size_t kk = (size_t)min(t, nst - 1) * 128;
    const uint32_t slot = lds_base + (uint32_t)((t % NS) * NBLK) * 1024u;
#pragma unroll
    for (int i = 0; i < PER; ++i) lds_dma16(src[i] + kk, slot + (uint32_t)(wave + 4 * i) * 1024u);
  };
  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) request(t);
  // EPI_QKV: the row's position depends on a loaded value (its cache length); it is turned into (slot, image index) only
  // now, behind the first stage requests, so that this wait is not on the path to them.  (Loads the compiler issues are
  // counted by the same counter as the stage loads: its waits and the hand-written ones below can only become stricter.)
  if (EPI == EPI_QKV) {
#pragma unroll
    for (int p = 0; p < RP; ++p) pre[p].start(tile_m * RP + p, tile_n, M, N, ep);
  }
  __builtin_amdgcn_sched_barrier(0);
  VVS_PHASE_MARK(1);
#define VVS_WAIT_STAGES asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER * (NS - 3)) : "memory")
  VVS_WAIT_STAGES;                         // stages 0 and 1 of this wave have landed
  __syncthreads();                         // ... and everybody else's
#define VVS_S2F(FA, FB, T, KBO)                                                                                       \
  {                                                                                                                   \
    const int sl = ((T) % NS) * NBLK;                                                                                 \
    _Pragma("unroll") for (int t = 0; t < WM; ++t)                                                                    \
        FA[t] = __builtin_bit_cast(bf16x8, stage[(sl + (wr * WM + t) * 2 + (KBO)) * 64 + lane]);                      \
    _Pragma("unroll") for (int t = 0; t < WN; ++t)                                                                    \
        FB[t] = __builtin_bit_cast(bf16x8, stage[(sl + NA + (wc * WN + t) * 2 + (KBO)) * 64 + lane]);                 \
  }
#define VVS_MMA(FA, FB)                                                                                               \
  {                                                                                                                   \
    _Pragma("unroll") for (int ti = 0; ti < WM; ++ti)                                                                 \
        _Pragma("unroll") for (int tj = 0; tj < WN; ++tj)                                                             \
            acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[ti], FB[tj], acc[ti][tj], 0, 0, 0);              \
  }
  bf16x8 fa0[WM], fb0[WN], fa1[WM], fb1[WN];
  VVS_S2F(fa0, fb0, 0, 0)
  // One stage = two groups of WM * WN MFMAs (contraction blocks 0 and 1).  A wave issues in order and an MFMA keeps its pipe
  // for 32 clocks, during which the wave may issue other kinds of instructions for free - but only if they stand BETWEEN
  // two MFMAs in program order.  So everything else a stage needs is dealt into the gaps, one or two items behind each MFMA:
  //   group A (fragments of block 0, read during the previous stage): the LDS reads of block 1 of this stage, then the
  //     stage requests for stage s + NS - 1 (into the slot stage s - 1 has left: everybody finished reading it before
  //     the last barrier);
  //   group B (block 1): the LDS reads of block 0 of stage s + 1 and, half way, the wait for this wave's part of stage
  //     s + 2 and the barrier - a bare s_barrier: the only LDS reads that must be complete before a slot is overwritten
  //     are those of stage s, and the MFMAs of group B have consumed them; waiting for the reads just issued (what
  //     __syncthreads would add) would drain the MFMA pipe once per stage.
  constexpr int NM = WM * WN, NR = WM + WN;
  constexpr int IA = (NR + PER + NM - 1) / NM;          // items per gap in group A
  constexpr int IB = (NR + NM - 1) / NM;                // items per gap in group B
  auto lds_frag = [&](int t, int kbo, int i) {           // i-th fragment of a stage's block kbo: A rows first, then B rows
    const int sl = (t % NS) * NBLK;
    return __builtin_bit_cast(bf16x8, stage[(sl + (i < WM ? (wr * WM + i) * 2 : NA + (wc * WN + (i - WM)) * 2) + kbo) * 64 + lane]);
  };
  for (int s = 0; s < nst; ++s) {
    const size_t kk = (size_t)min(s + NS - 1, nst - 1) * 128;
    const uint32_t slot = lds_base + (uint32_t)(((s + NS - 1) % NS) * NBLK) * 1024u;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      acc[m / WN][m % WN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0[m / WN], fb0[m % WN], acc[m / WN][m % WN], 0, 0, 0);
#pragma unroll
      for (int it = m * IA; it < (m + 1) * IA; ++it) {
        if (it < NR) {
          if (it < WM) fa1[it] = lds_frag(s, 1, it); else fb1[it - WM] = lds_frag(s, 1, it);
        } else if (it - NR < PER) {
          const int i = it - NR;
          lds_dma16(src[i] + kk, slot + (uint32_t)(wave + 4 * i) * 1024u);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      acc[m / WN][m % WN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1[m / WN], fb1[m % WN], acc[m / WN][m % WN], 0, 0, 0);
#pragma unroll
      for (int it = m * IB; it < (m + 1) * IB; ++it) {
        if (it < NR) {
          if (it < WM) fa0[it] = lds_frag(s + 1, 0, it); else fb0[it - WM] = lds_frag(s + 1, 0, it);
        }
      }
      if (m == NM / 2) {
        VVS_WAIT_STAGES;                   // this wave's part of stage s + 2
        __builtin_amdgcn_s_barrier();      // ... and everybody else's; and everybody is done reading stage s
        asm volatile("" ::: "memory");
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#undef VVS_MMA
#undef VVS_S2F
  VVS_PHASE_MARK(2);
#pragma unroll
  for (int p = 0; p < RP; ++p) pre[p].to_lds(s_pos + p * 2 * EM, nullptr, ep);
  rowscale.finish(rs, tile_m, M, ep);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the repeated last stages still in flight must land before the tile reuses their LDS
#undef VVS_WAIT_STAGES
  __syncthreads();                         // the stage buffers become the output tile
#pragma unroll
  for (int p = 0; p < RP; ++p) {
    if (RP == 1 || wr == p) {              // RP == 2: pass p holds the rows of wave row p
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            red[(((RP == 1 ? wr * WM : 0) + i) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * LDC + (wc * WN + j) * 32 + (lane & 31)] = acc[i][j][r];
    }
    __syncthreads();
    VVS_PHASE_MARK(3);
    tile_epilogue<EM, BN, 1, EPI, EARLY>(red, rs + p * EM, tile_m * RP + p, tile_n, M, N, C, ep, pre[p], s_pos + p * 2 * EM, nullptr);
    if (p + 1 < RP) __syncthreads();       // the next pass overwrites the tile
  }
  VVS_PHASE_MARK(4);
}

template <int WM, int WN, int NS, int EPI>
static void launch_gemm_shared_dma(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, const GemmEpi& ep, hipStream_t s) {
  constexpr int BM = 2 * WM * 32, BN = 2 * WN * 32;
  constexpr size_t lds_full = (size_t)BM * (BN + 4) * sizeof(float), lds_tile = lds_full > 140 * 1024 ? lds_full / 2 : lds_full;   // two passes
  constexpr size_t lds_stage = (size_t)NS * (2 * (BM + BN) / 32) * 1024;
  constexpr size_t lds = lds_tile > lds_stage ? lds_tile : lds_stage;
  allow_dynamic_lds(reinterpret_cast<const void*>(&k_gemm_shared_dma<WM, WN, NS, EPI>), lds);
  dim3 grid((N / BN) * ((M + BM - 1) / BM), 1, 1);
  hipLaunchKernelGGL((k_gemm_shared_dma<WM, WN, NS, EPI>), grid, dim3(256), lds, s, (const uint4*)A, (const uint4*)W, C, M, N, K, ep);
}

template <int WM, int WN, int D, int EPI>
static void launch_gemm_shared(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, const GemmEpi& ep, hipStream_t s) {
  constexpr int BM = 2 * WM * 32, BN = 2 * WN * 32;
  constexpr size_t lds_tile = (size_t)BM * (BN + 4) * sizeof(float), lds_stage = (size_t)3 * (2 * (BM + BN) / 32) * 1024;
  constexpr size_t lds = lds_tile > lds_stage ? lds_tile : lds_stage;
  allow_dynamic_lds(reinterpret_cast<const void*>(&k_gemm_shared<WM, WN, D, EPI>), lds);
  dim3 grid((N / BN) * ((M + BM - 1) / BM), 1, 1);
  hipLaunchKernelGGL((k_gemm_shared<WM, WN, D, EPI>), grid, dim3(256), lds, s, (const uint4*)A, (const uint4*)W, C, M, N, K, ep);
}

template <int TM, int TN, int D, int EPI>
static void launch_gemm_direct(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, int splits, const GemmEpi& ep,
                               hipStream_t s) {
  constexpr size_t lds = (size_t)4 * TM * 32 * (TN * 32 + 4) * sizeof(float);
  allow_dynamic_lds(reinterpret_cast<const void*>(&k_gemm_direct<TM, TN, D, EPI>), lds);
  const int KB = K / 16;
  const int per = (KB + splits - 1) / splits;
  dim3 grid((N / (TN * 32)) * ((M + TM * 32 - 1) / (TM * 32)), 1, splits);
  hipLaunchKernelGGL((k_gemm_direct<TM, TN, D, EPI>), grid, dim3(256), lds, s, (const uint4*)A, (const uint4*)W, C, M, N, K, per, ep);
}

template <int EPI>
static void gemm_dispatch(const bf16_t* A, const bf16_t* W, float* C, int M, int N, int K, GemmPlan p, const GemmEpi& ep, hipStream_t s) {
  if constexpr (EPI != EPI_RESID) {
    // very many rows: 256 x 256 tiles (128 x 128 per wave, the accumulators fill the 256 AGPRs; half the operand bytes per
    // flop of a 128 x 128 tile come through a CU's L1), when they give (nearly) every CU a tile.  EPI_QKV: a tile must lie
    // inside one of the q / k / v thirds.
    const int t256 = ((M + 255) / 256) * (N / 256);
    if (p.bm == 128 && p.bn == 128 && N % 256 == 0 && t256 >= 224 && (EPI != EPI_QKV || ep.d % 256 == 0)) {
      launch_gemm_shared_dma<4, 4, 4, EPI>(A, W, C, M, N, K, ep, s);
      return;
    }
  }
  if constexpr (EPI == EPI_QKV) {
    // many rows (two or more full rounds of 128 x 128 tiles): the direct-to-LDS kernel, two workgroups per CU
    const int tiles = ((M + 127) / 128) * (N / 128);
    if (p.bm == 128 && p.bn == 128 && tiles >= 512) { launch_gemm_shared_dma<2, 2, 4, EPI>(A, W, C, M, N, K, ep, s); return; }
  }
  if constexpr (EPI == EPI_PARTIAL || EPI == EPI_SWIGLU) {
    // the stages are loaded straight into LDS.  A single round of tiles (at most one workgroup per CU): 8 slots, 6
    // stages in flight.  Two or more full rounds: 4 slots, so that the LDS (the 68 KB of the output tile) lets two
    // workgroups share a CU and cover each other's barrier waits.  In between (257 .. 511 tiles) the variant that
    // stages through registers is the faster one (384 tiles: 28 against 32 us).
    const int tiles = ((M + 127) / 128) * (N / 128);
    if (p.bm == 128 && p.bn == 128 && tiles <= 256) { launch_gemm_shared_dma<2, 2, 8, EPI>(A, W, C, M, N, K, ep, s); return; }
    if (p.bm == 128 && p.bn == 128 && tiles >= 512) { launch_gemm_shared_dma<2, 2, 4, EPI>(A, W, C, M, N, K, ep, s); return; }
  }
  if constexpr (EPI != EPI_RESID) {
    if (p.bm == 128 && p.bn == 128) { launch_gemm_shared<2, 2, 6, EPI>(A, W, C, M, N, K, ep, s); return; }
  }
  if (p.bm == 32 && p.bn == 128) launch_gemm_direct<1, 4, 4, EPI>(A, W, C, M, N, K, p.splits, ep, s);
  else if (p.bm == 32) launch_gemm_direct<1, 2, 8, EPI>(A, W, C, M, N, K, p.splits, ep, s);
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

// x += A W; also leaves bf16(x * g_next) packed and the per-slab sums of squares of the new x
void mfma_gemm_resid(Ctx* c, const bf16_t* A, const bf16_t* W, float* x, bf16_t* xb, float* ss_out, const float* g_next, int M, int K,
                     hipStream_t s, int xb_T, int xb_pad) {
  GemmEpi ep{};
  ep.x = x; ep.xb = xb; ep.ss_out = ss_out; ep.g_next = g_next; ep.NS = (c->d / 64 + 3) & ~3; ep.xb_T = xb_T; ep.xb_pad = xb_pad;
  // many rows: 192 x 128 tiles with the operands shared through LDS (a quarter of the bytes per flop that 64 x 64 tiles pull
  // through a CU's L1), when they give most CUs a tile - at d = 1280 and 3904 rows: 210 tiles, one round
  if (c->d % 128 == 0 && K % 32 == 0 && ((M + 191) / 192) * (c->d / 128) >= 160) {
    // fabric traffic of the two tile orders: the operand an XCD does not own is fetched by all 8 of them
    ep.row_owner = (size_t)M + 8 * (size_t)c->d < 8 * (size_t)M + (size_t)c->d;
    launch_gemm_shared_dma<3, 2, 6, EPI_RESID>(A, W, nullptr, M, c->d, K, ep, s);
    return;
  }
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

// One 32-key step of the attention kernels for NQB blocks of 16 queries: scores S^T = K Q^T (lane = query l % 16, key
// group g = l / 16, 8 consecutive keys per lane), online softmax, O^T += V^T P^T.  The tree mask only touches a step that
// reaches past the cached length S (tail).
// The softmax weights are not rounded to bf16 (the definition keeps them exact): each un-normalised weight e goes into the
// P V product as the sum of two bf16 values, hi = bf16(e) and lo = bf16(e - hi) (e to 2^-17), with two MFMAs per V block -
// the matrix cores idle in these kernels anyway - and the normaliser sums the fp32 weights themselves.
template <int NQB, int KD, int DT>
__device__ __forceinline__ void attn_step(const bf16x8 (&kf)[2][KD], const bf16x8 (&vf)[DT], const bf16x8 (&qf)[NQB][KD],
                                          const uint64_t (&mask)[NQB], float (&m_run)[NQB], float (&l_run)[NQB], floatx4 (&o)[NQB][DT],
                                          int key0, int S, int n_keys, bool tail, int g, float c_exp) {
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
    mx = rows_max(mx);
    const float m_new = fmaxf(m_run[qb], mx);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_safe) * c_exp);
    const float mc = m_safe * c_exp;
    uint32_t pk[4], pl[4];
    float rs = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
      // hardware exp2 (arguments <= 0 up to the rounding of the fused multiply-add)
      const float e0 = __builtin_amdgcn_exp2f(fmaf(sv[i], c_exp, -mc)), e1 = __builtin_amdgcn_exp2f(fmaf(sv[i + 1], c_exp, -mc));
      const uint32_t pp = pack2bf(e0, e1);
      rs += e0 + e1;
      pk[i >> 1] = pp;
      pl[i >> 1] = pack2bf(e0 - __uint_as_float(pp << 16), e1 - __uint_as_float(pp & 0xFFFF0000u));
    }
    rs = rows_sum(rs);
    l_run[qb] = l_run[qb] * alpha + rs;
    m_run[qb] = m_new;
    const bf16x8 pf = as_bf16x8(make_uint4(pk[0], pk[1], pk[2], pk[3]));
    const bf16x8 pfl = as_bf16x8(make_uint4(pl[0], pl[1], pl[2], pl[3]));
    // the running maximum rarely moves after the first steps: the accumulators are only rescaled when some query's did
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) o[qb][dt][rr] *= alpha;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      o[qb][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf, o[qb][dt], 0, 0, 0);
      o[qb][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pfl, o[qb][dt], 0, 0, 0);
    }
  }
}

// ------------------------------------------------------------------------------------------------ attention
// One workgroup per (head, row).  Scores are computed transposed, S^T[key][query] = K * Q^T, so the
// accumulator layout (lane = query, registers = keys) is directly the B operand of
// O^T[dim][query] = V^T[dim][key] * P^T[key][query] and the online-softmax state of a query lives in
// one lane.  The cache keeps K and V in the operand order of these MFMAs (k_index / v_index), so they
// are loaded straight into operand registers with fully contiguous wave-wide loads - every key is used
// by exactly one wave, so there is nothing to share through LDS; the 4 waves take 32-key steps
// round-robin and merge their partial (max, sum, O) through LDS at the end.  Only the last T keys (the
// block itself) are masked.
// QG > 1: the queries are dealt to QG groups of NW waves (group g takes queries g * NQB * 16 ...); every group runs over all
// keys.  More than 32 queries per wave need more registers than leave room for a second workgroup on the CU, and a
// lone workgroup pays its start-up (first requests, merge) with nothing to cover it; two groups of 32 queries keep
// three workgroups resident, and the second group's K/V requests mostly hit the lines the first one brought in.
template <int DH, int NQB, int NW, int PD, int QG = 1>
__global__ __launch_bounds__(NW * QG * 64, (DH * NQB >= 256 ? 1 : 2)) void k_attn_mfma(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc,
                                                   const bf16_t* __restrict__ vc, bf16_t* __restrict__ out, TreeDesc tree,
                                                   PosDesc pos, int T, int d, size_t row_stride, size_t head_stride, float c_exp,
                                                   int cap_steps) {
  constexpr int KD = DH / 32, DT = DH / 16, NQ = NQB * 16;
  __shared__ float s_m[QG][NW - 1][NQ], s_l[QG][NW - 1][NQ];
  __shared__ float s_o[QG][NW - 1][NQ][DH + 1];
  VVS_PHASE_MARK(0);
  const int hd = blockIdx.x, r = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) % NW, qg = (threadIdx.x >> 6) / NW, q0 = qg * NQ;
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
    // query rows past T repeat row T - 1: a query only ever touches its own lanes' columns and rows >= T
    // are not stored, so nothing has to be zeroed - and no load result is needed before the first MFMA
    const int tq = min(q0 + qb * 16 + ql, T - 1);
    mask[qb] = tree.anc[tq];
#pragma unroll
    for (int kd = 0; kd < KD; ++kd)
      qf[qb][kd] = as_bf16x8(*(const uint4*)(q + ((size_t)r * T + tq) * d + (size_t)hd * DH + kd * 32 + g * 8));
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

  // K and V of one 32-key step, straight into MFMA operand registers: the cache is kept in operand
  // order (k_index / v_index), so every load instruction of a wave reads 1 KiB of contiguous memory.
  // S^T tile t, row i holds key 8*(i/4) + 4*t + i%4 of the step: a lane's 8 score values are 8 consecutive keys.
#define VVS_ATTN_LOAD(STEP, KF, VF)                                                                                   \
  {                                                                                                                   \
    _Pragma("unroll") for (int t = 0; t < 2; ++t)                                                                     \
        _Pragma("unroll") for (int kd = 0; kd < KD; ++kd)                                                             \
            KF[t][kd] = as_bf16x8(*(const uint4*)(kb + ((((size_t)(STEP) * 2 + t) * KD + kd) * 64 + lane) * 8));      \
    _Pragma("unroll") for (int dt = 0; dt < DT; ++dt)                                                                 \
        VF[dt] = as_bf16x8(*(const uint4*)(vb + (((size_t)(STEP) * DT + dt) * 64 + lane) * 8));                       \
  }
  // Ring of PD operand sets: a wave's steps wave, wave + NW, ... ; the operands of a step are requested
  // PD steps ahead, right after the set's previous step has been multiplied, so that the cache streams
  // in while the wave computes.  Requests past the row's last step repeat that step (never used).
  bf16x8 kf[PD][2][KD], vf[PD][DT];
#pragma unroll
  for (int p = 0; p < PD; ++p) {
    // first requests: clamped to the cache capacity, not to the row's length, so that their addresses do
    // not wait for the length (a memory read); steps past the end are valid memory that is never used
    VVS_ATTN_LOAD(min(wave + p * NW, cap_steps - 1), kf[p], vf[p]);
    __builtin_amdgcn_sched_barrier(0);               // request groups stay in program order: waits are partial
  }
  VVS_PHASE_MARK(1);
  for (int base = wave; base < nsteps; base += NW * PD) {
#pragma unroll
    for (int p = 0; p < PD; ++p) {
      const int step = base + p * NW;
      if (step < nsteps) {
        const int key0 = step << 5;
        const bool tail = key0 + 32 > S;
        attn_step<NQB, KD, DT>(kf[p], vf[p], qf, mask, m_run, l_run, o, key0, S, n_keys, tail, g, c_exp);
      }
      VVS_ATTN_LOAD(min(step + PD * NW, nsteps - 1), kf[p], vf[p]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#undef VVS_ATTN_LOAD

  VVS_PHASE_MARK(2);
  // merge the waves' partial results (waves 1.. publish, wave 0 combines and writes)
  if (wave > 0) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int qi = qb * 16 + ql;
      if (g == 0) { s_m[qg][wave - 1][qi] = m_run[qb]; s_l[qg][wave - 1][qi] = l_run[qb]; }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) s_o[qg][wave - 1][qi][dt * 16 + 4 * g + rr] = o[qb][dt][rr];
    }
  }
  __syncthreads();
  VVS_PHASE_MARK(3);
  if (wave == 0) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int qi = qb * 16 + ql;
      float m = m_run[qb];
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) m = fmaxf(m, s_m[qg][w][qi]);
      const float m_safe = m == -INFINITY ? 0.f : m;
      const float a0 = exp2f((m_run[qb] - m_safe) * c_exp);
      float l = l_run[qb] * a0;
      float aw[NW - 1];
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) {
        aw[w] = exp2f((s_m[qg][w][qi] - m_safe) * c_exp);
        l += s_l[qg][w][qi] * aw[w];
      }
      const float inv = 1.0f / l;
      if (q0 + qi < T) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          uint32_t pk[2];
#pragma unroll
          for (int rr = 0; rr < 4; rr += 2) {
            float v0 = o[qb][dt][rr] * a0, v1 = o[qb][dt][rr + 1] * a0;
#pragma unroll
            for (int w = 0; w < NW - 1; ++w) {
              v0 += s_o[qg][w][qi][dt * 16 + 4 * g + rr] * aw[w];
              v1 += s_o[qg][w][qi][dt * 16 + 4 * g + rr + 1] * aw[w];
            }
            pk[rr >> 1] = pack2bf(v0 * inv, v1 * inv);
          }
          *(uint2*)(out + pack_index(r * T + q0 + qi, hd * DH + dt * 16 + 4 * g, d)) = make_uint2(pk[0], pk[1]);   // O-projection operand layout
        }
      }
    }
  }
  VVS_PHASE_MARK(4);
}

// ------------------------------------------------------------------------------------------------ q/k/v projection + attention in one launch
// Verify calls with at most 64 block tokens per row and head size 64: one workgroup per (head, prompt) computes the head's
// q, k and v columns for the prompt's two rows (conditional, unconditional) and goes straight on to their attention, so that
// the layer has one launch less and attention does not start from a cold ramp of its own: q never leaves the CU, and k / v
// are read back from the cache lines the same workgroup has just written.
//   TR = 32 or 64: tile rows per row of the pair (T <= TR).
//   Projection: a (2 TR) x 192 tile on the direct-to-LDS pipeline of k_gemm_shared_dma (2 x 2 waves of TR x 96; a stage = 32
//     contraction values = 16 or 20 KiB).  The activation operand comes in the ROW-PADDED packed layout - row r starts at
//     packed row r * TR, so the tile's row-blocks are those of rows 2b and 2b + 1 - and the weight blocks are the head's two
//     32-row blocks inside each of the q, k and v thirds.  Tile rows t >= T are padding: every output row depends on its
//     own operand row only, and those rows are never used.
//   Epilogue: RMSNorm row factor, 2D rotary embedding of q and k; q goes to LDS (bf16), k and v into their cache slots.
//   Attention: as k_attn_mfma with four waves per (head, row) - the workgroup has 8 waves: waves 0-3 run the projection,
//     then even waves take the conditional row and odd waves the unconditional one - reading q fragments from LDS.  With
//     TR = 64 a row's waves form two groups of two, one per 32 queries (64 queries per wave would not fit the registers).
//     Waves 4-7 have no MFMAs during the projection: they take their share of the stage requests (TR = 32) and meet the
//     barriers, and when the last stage has landed they request the K / V operands of their first steps, where those steps
//     lie wholly below the cache length (old keys), so that these arrive while the tile goes through the epilogue.  Every
//     other cache load stands behind the workgroup-scope fence and the barrier that follow the cache writes, and no line
//     holding a slot of the block itself is read before them, so the L1 of the CU cannot hold a stale copy of the slots
//     just written.
//   Measured with time stamps at the end of the image (TR = 32, 55 k cycles): start-up 3 k, projection main loop 24 k (16 KiB
//     per 600 cycles, paced by how fast the CU's address unit takes the stage requests: without them the loop takes 4.4 of
//     its 10.4 us, without the MFMAs 10.2), tile to LDS 2.5 k, epilogue + fence 5 k, attention steps 17 k, merge + store 3 k.
template <int NSL, int TR, int NQB>
__global__ __launch_bounds__(512) void k_qkv_attn(const uint4* __restrict__ Ap, const uint4* __restrict__ Wp, bf16_t* __restrict__ out,
                                                  int K, const GemmEpi ep, float c_exp) {
  constexpr int GW = 4;                    // projection waves: 2 x 2 of TR x 96 (1 x 2 of 64 x 96 at TR = 32 measured 3 % slower per step)
  constexpr int RB = TR / 32;              // 32-row blocks per row of the pair
  constexpr int WM = RB, WN = 3, BM = 2 * TR, BN = 192, LDC = BN + 4, NA = 2 * (BM / 32), NBLK = NA + 12;
  constexpr int DW = NBLK % 8 == 0 ? 8 : 4;   // waves that request stage blocks (the projection waves among them)
  constexpr int PER = NBLK / DW;
  static_assert(TR == 32 || TR == 64, "one or two row-blocks per row");
  static_assert(NBLK % DW == 0, "stage blocks are dealt to the requesting waves");
  constexpr int DH = 64, KD = DH / 32, DT = DH / 16, NQ = NQB * 16, PD = 2;
  constexpr int QG = RB, NW = 4 / QG;      // query groups of 32 per row, waves per group
  static_assert(NQ * QG >= TR || (TR == 32 && NQB == 1), "every query has a lane");
  constexpr int QLD = DH + 8;              // bf16 per q row in LDS: 144 bytes, 16-byte aligned, rows spread over the banks
  constexpr size_t kRing = (size_t)NSL * NBLK * 1024, kTile = (size_t)BM * LDC * sizeof(float);
  constexpr size_t kFirst = kRing > kTile ? kRing : kTile;
  static_assert(NSL >= 4 && PER * (NSL - 1) <= 60, "stages in flight / 6-bit load counter");
  static_assert(kFirst >= (size_t)2 * 4 * NQ * (DH + 3) * sizeof(float), "the merge buffers reuse the tile");
  extern __shared__ float red[];           // stage ring, then the output tile, then the attention merge buffers; behind it q
  u32x4* stage = (u32x4*)red;
  bf16_t* q_s = (bf16_t*)((char*)red + kFirst);                // [2 rows][TR tokens][QLD]
  float* s_o = red;                                            // [2 rows][4 waves][NQ][DH + 1]
  float* s_m = s_o + 2 * 4 * NQ * (DH + 1);                    // [2 rows][4 waves][NQ]
  float* s_l = s_m + 2 * 4 * NQ;
  __shared__ float rs[BM];
  const uint32_t lds_base = (uint32_t)(uintptr_t)stage;
  VVS_PHASE_MARK(0);
  const int hd = blockIdx.x, b = blockIdx.y, T = ep.T, d = ep.d;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool gemm_wave = wave < GW, dma_wave = wave < DW;
  const bool rs_thread = (int)threadIdx.x < BM * 4;   // the threads that own the row factors: 4 lanes per tile row
  const int wr = (wave >> 1) & 1, wc = wave & 1;
  // attention: row of the pair, wave within the row (each row: two projection waves, two others), query group, wave within the group
  const int ar = wave & 1, ai = wave >> 1, qg = ai / NW, aw = ai % NW, q0 = qg * 32;
  const int KB = K >> 4, nst = KB >> 1;
  // The prompt's cache length and emitted count come from memory (a scalar load that shares its counter with the
  // kernel-argument loads): they are asked for only behind the first stage requests, so that nothing on the way to those
  // requests waits for memory.
  int kv, ne;
  float4 rv[4];                            // row factor inputs
  // attention operands (see k_attn_mfma): K and V of a 32-key step straight into MFMA operand registers
  const int r = 2 * b + ar;
  const int g = lane >> 4, ql = lane & 15;
  const int cap_steps = ep.S_cap >> 5;
  const bf16_t* kb = ep.kc + (size_t)r * ep.row_stride + (size_t)hd * ep.head_stride;
  const bf16_t* vb = ep.vc + (size_t)r * ep.row_stride + (size_t)hd * ep.head_stride;
#define VVS_ATTN_LOAD(STEP, KF, VF)                                                                                   \
  {                                                                                                                   \
    _Pragma("unroll") for (int t = 0; t < 2; ++t)                                                                     \
        _Pragma("unroll") for (int kd = 0; kd < KD; ++kd)                                                             \
            KF[t][kd] = as_bf16x8(*(const uint4*)(kb + ((((size_t)(STEP) * 2 + t) * KD + kd) * 64 + lane) * 8));      \
    _Pragma("unroll") for (int dt = 0; dt < DT; ++dt)                                                                 \
        VF[dt] = as_bf16x8(*(const uint4*)(vb + (((size_t)(STEP) * DT + dt) * 64 + lane) * 8));                       \
  }
  bf16x8 kf[PD][2][KD], vf[PD][DT];
  bool early[PD];
  floatx16 acc[WM][WN];
  if (rs_thread) {                         // row factor inputs (as RowScale): each lane every 4th group of 4 slabs; addresses from
    const int row = threadIdx.x >> 2, part = threadIdx.x & 3, nq = ep.NS >> 2;   // kernel arguments only, older than the stage requests
    const int m = (2 * b + row / TR) * T + min(row % TR, T - 1);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      rv[i] = part + 4 * i < nq ? ((const float4*)(ep.ss + (size_t)m * ep.NS))[part + 4 * i] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __builtin_amdgcn_sched_barrier(0);
  const u32x4* src[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int j = min(wave + DW * i, NBLK - 1);   // block of the stage: 0 .. NA-1 activations (row-block, contraction half), then 12 weight blocks
    const int wi = (j - NA) >> 1;          // weight block: third (q, k, v) = wi / 2, half of the head = wi % 2
    const int rb = j < NA ? 2 * b * RB + (j >> 1) : (wi >> 1) * (d >> 5) + 2 * hd + (wi & 1);
    src[i] = (const u32x4*)(j < NA ? Ap : Wp) + ((size_t)rb * KB + (j & 1)) * 64 + lane;
  }
  auto request = [&](int t) {
    const size_t kk = (size_t)min(t, nst - 1) * 128;
    const uint32_t slot = lds_base + (uint32_t)((t % NSL) * NBLK) * 1024u;
#pragma unroll
    for (int i = 0; i < PER; ++i) lds_dma16(src[i] + kk, slot + (uint32_t)(wave + DW * i) * 1024u);
  };
  if (dma_wave) {
#pragma unroll
    for (int t = 0; t < NSL - 1; ++t) request(t);
  }
  __builtin_amdgcn_sched_barrier(0);
  VVS_PHASE_MARK(1);
  kv = ep.pos.kv_len[b];
  ne = ep.pos.n_emitted[b];
#pragma unroll
  for (int p = 0; p < PD; ++p) early[p] = false;
  __builtin_amdgcn_sched_barrier(0);
#define VVS_WAIT_STAGES asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER * (NSL - 3)) : "memory")
  if (gemm_wave) {
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) acc[i][j][rr] = 0.f;
    VVS_WAIT_STAGES;                       // stages 0 and 1 of this wave have landed
    __syncthreads();                       // ... and everybody else's
    constexpr int NM = WM * WN, NR = WM + WN;
    constexpr int IA = (NR + PER + NM - 1) / NM, IB = (NR + NM - 1) / NM;
    auto lds_frag = [&](int t, int kbo, int i) {         // i-th fragment of a stage's block kbo: the A row-blocks first, then the B blocks
      const int sl = (t % NSL) * NBLK;
      return __builtin_bit_cast(bf16x8, stage[(sl + (i < WM ? (wr * WM + i) * 2 : NA + (wc * WN + (i - WM)) * 2) + kbo) * 64 + lane]);
    };
    bf16x8 fa0[WM], fb0[WN], fa1[WM], fb1[WN];
#pragma unroll
    for (int i = 0; i < WM; ++i) fa0[i] = lds_frag(0, 0, i);
#pragma unroll
    for (int j = 0; j < WN; ++j) fb0[j] = lds_frag(0, 0, WM + j);
    // the main loop of k_gemm_shared_dma: everything but the MFMAs is dealt into the gaps between them
    for (int s = 0; s < nst; ++s) {
      const size_t kk = (size_t)min(s + NSL - 1, nst - 1) * 128;
      const uint32_t slot = lds_base + (uint32_t)(((s + NSL - 1) % NSL) * NBLK) * 1024u;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        acc[m / WN][m % WN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0[m / WN], fb0[m % WN], acc[m / WN][m % WN], 0, 0, 0);
#pragma unroll
        for (int it = m * IA; it < (m + 1) * IA; ++it) {
          if (it < NR) {
            if (it < WM) fa1[it] = lds_frag(s, 1, it); else fb1[it - WM] = lds_frag(s, 1, it);
          } else if (it - NR < PER) {
            const int i = it - NR;
            lds_dma16(src[i] + kk, slot + (uint32_t)(wave + DW * i) * 1024u);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        acc[m / WN][m % WN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1[m / WN], fb1[m % WN], acc[m / WN][m % WN], 0, 0, 0);
#pragma unroll
        for (int it = m * IB; it < (m + 1) * IB; ++it) {
          if (it < NR) {
            if (it < WM) fa0[it] = lds_frag(s + 1, 0, it); else fb0[it - WM] = lds_frag(s + 1, 0, it);
          }
        }
        if (m == NM / 2) {
          VVS_WAIT_STAGES;                 // this wave's part of stage s + 2
          __builtin_amdgcn_s_barrier();    // ... and everybody else's; and everybody is done reading stage s
          asm volatile("" ::: "memory");
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the repeated last stages still in flight must land before the tile reuses their LDS
  } else {                                 // the other waves: their share of the stage requests and the barriers of the main loop
    if (dma_wave) VVS_WAIT_STAGES;
    __syncthreads();
    for (int s = 0; s < nst; ++s) {
      if (dma_wave) {                      // into the slot stage s - 1 has left: everybody finished reading it before the last barrier
        request(s + NSL - 1);
        VVS_WAIT_STAGES;
      }
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    }
    if (dma_wave) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // before the tile reuses the ring
    // the K / V operands of this wave's first steps, where they lie wholly below the cache length (old keys only): they
    // arrive while the tile goes through the epilogue
#pragma unroll
    for (int p = 0; p < PD; ++p) {
      early[p] = aw + p * NW < (kv >> 5);  // wave-uniform
      if (early[p]) VVS_ATTN_LOAD(aw + p * NW, kf[p], vf[p]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const int S = kv, n_keys = S + T, nsteps = (n_keys + 31) >> 5;
  if (rs_thread) {                         // row factors
    const int row = threadIdx.x >> 2, part = threadIdx.x & 3;
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) t += (rv[i].x + rv[i].y) + (rv[i].z + rv[i].w);
    t += __shfl_xor(t, 1, 64);
    t += __shfl_xor(t, 2, 64);
    if (part == 0) rs[row] = 1.0f / sqrtf(t / (float)ep.dnorm + ep.eps);
  }
#undef VVS_WAIT_STAGES
  VVS_PHASE_MARK(2);
  __syncthreads();                         // the stage buffers become the output tile
  if (gemm_wave) {
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int rr = 0; rr < 16; ++rr)
          red[((wr * WM + i) * 32 + (rr >> 2) * 8 + (lane >> 5) * 4 + (rr & 3)) * LDC + (wc * WN + j) * 32 + (lane & 31)] = acc[i][j][rr];
  }
  __syncthreads();
  VVS_PHASE_MARK(3);

  // ---- epilogue: tile columns 0..63 q, 64..127 k, 128..191 v of head hd; tile row = TR * (row of the pair) + token
  constexpr int np = DH >> 2, half = DH >> 1;   // rotary pairs per grid axis; dims of the grid-row half
#pragma unroll
  for (int u = threadIdx.x; u < BM * 4; u += 512) {     // q: one unit = (tile row, 16 consecutive dims)
    const int row = u >> 2, c0 = (u & 3) * 16, t = row % TR;
    if (t < T) {
      const float4* p4 = (const float4*)(red + row * LDC + c0);
      const float4 s0 = p4[0], s1 = p4[1], s2 = p4[2], s3 = p4[3];
      float v[16] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w, s2.x, s2.y, s2.z, s2.w, s3.x, s3.y, s3.z, s3.w};
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] *= rs[row];
      const int img = ne - 1 + ep.tree.depth[t];
      if (img >= 0) {
        const int gr = min(img / ep.pos.grid_w, ep.rope_pos - 1), gc = img % ep.pos.grid_w;
        // 16 dims = 8 pairs inside one half of the head: 8 consecutive pairs of one table row
        const float4* t4 = (const float4*)(ep.rope + ((size_t)(c0 >= half ? gc : gr) * np + ((c0 & (half - 1)) >> 1)) * 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float4 c4 = t4[i];
          const float a0 = v[4 * i], b0 = v[4 * i + 1], a1 = v[4 * i + 2], b1 = v[4 * i + 3];
          v[4 * i] = a0 * c4.x - b0 * c4.y;
          v[4 * i + 1] = a0 * c4.y + b0 * c4.x;
          v[4 * i + 2] = a1 * c4.z - b1 * c4.w;
          v[4 * i + 3] = a1 * c4.w + b1 * c4.z;
        }
      }
      uint4* dst = (uint4*)(q_s + row * QLD + c0);
      dst[0] = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
      dst[1] = make_uint4(pack2bf(v[8], v[9]), pack2bf(v[10], v[11]), pack2bf(v[12], v[13]), pack2bf(v[14], v[15]));
    }
  }
  // k and v: a lane takes one tile row (token), the lanes of a wave consecutive tokens
#pragma unroll
  for (int u = threadIdx.x; u < BM * 8; u += 512) {     // k: one unit = (tile row, 8 dims), one 16-byte store each
    const int row = u % BM, c8 = (u / BM) * 8, t = row % TR;
    const int slot = kv + t;
    if (t < T && slot >= 0 && slot < ep.S_cap) {
      const float sc = rs[row];
      bf16_t* kh = ep.kc + (size_t)(2 * b + row / TR) * ep.row_stride + (size_t)hd * ep.head_stride;
      const int img = ne - 1 + ep.tree.depth[t];
      const float4 a = *(const float4*)(red + row * LDC + DH + c8), bq = *(const float4*)(red + row * LDC + DH + c8 + 4);
      float v[8] = {a.x * sc, a.y * sc, a.z * sc, a.w * sc, bq.x * sc, bq.y * sc, bq.z * sc, bq.w * sc};
      if (img >= 0) {
        const int gr = min(img / ep.pos.grid_w, ep.rope_pos - 1), gc = img % ep.pos.grid_w;
        const float4* t4 = (const float4*)(ep.rope + ((size_t)(c8 >= half ? gc : gr) * np + ((c8 & (half - 1)) >> 1)) * 2);
        const float4 c0 = t4[0], c1 = t4[1];
        const float x0 = v[0], x1 = v[1], x2 = v[2], x3 = v[3], x4 = v[4], x5 = v[5], x6 = v[6], x7 = v[7];
        v[0] = x0 * c0.x - x1 * c0.y; v[1] = x0 * c0.y + x1 * c0.x;
        v[2] = x2 * c0.z - x3 * c0.w; v[3] = x2 * c0.w + x3 * c0.z;
        v[4] = x4 * c1.x - x5 * c1.y; v[5] = x4 * c1.y + x5 * c1.x;
        v[6] = x6 * c1.z - x7 * c1.w; v[7] = x6 * c1.w + x7 * c1.z;
      }
      *(uint4*)(kh + k_index(slot, c8, DH)) = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
    }
  }
#pragma unroll
  for (int u = threadIdx.x; u < BM * 16; u += 512) {    // v: one unit = (tile row, 4 dims); a store instruction covers runs of consecutive slots
    const int row = u % BM, c4 = (u / BM) * 4, t = row % TR;
    const int slot = kv + t;
    if (t < T && slot >= 0 && slot < ep.S_cap) {
      const float sc = rs[row];
      bf16_t* vh = ep.vc + (size_t)(2 * b + row / TR) * ep.row_stride + (size_t)hd * ep.head_stride;
      const float4 v = *(const float4*)(red + row * LDC + 2 * DH + c4);
      vh[v_index(slot, c4, DH)] = f2bf(v.x * sc);
      vh[v_index(slot, c4 + 1, DH)] = f2bf(v.y * sc);
      vh[v_index(slot, c4 + 2, DH)] = f2bf(v.z * sc);
      vh[v_index(slot, c4 + 3, DH)] = f2bf(v.w * sc);
    }
  }
  // the cache writes have reached L2 (the L1 is write-through) and q is in LDS before anybody goes on
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __syncthreads();
  VVS_PHASE_MARK(4);

  // ---- attention of (head hd, row 2b + ar), queries q0 .. q0 + NQ - 1, by the NW waves of the group (see k_attn_mfma)
  bf16x8 qf[NQB][KD];
  uint64_t mask[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int tq = min(q0 + qb * 16 + ql, T - 1);      // query rows past T repeat row T - 1 and are not stored
    mask[qb] = ep.tree.anc[tq];
#pragma unroll
    for (int kd = 0; kd < KD; ++kd) qf[qb][kd] = as_bf16x8(*(const uint4*)(q_s + (ar * TR + tq) * QLD + kd * 32 + g * 8));
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
#pragma unroll
  for (int p = 0; p < PD; ++p) {
    if (!early[p]) VVS_ATTN_LOAD(min(aw + p * NW, cap_steps - 1), kf[p], vf[p]);
    __builtin_amdgcn_sched_barrier(0);
  }
  for (int base = aw; base < nsteps; base += NW * PD) {
#pragma unroll
    for (int p = 0; p < PD; ++p) {
      const int step = base + p * NW;
      if (step < nsteps) {
        const int key0 = step << 5;
        const bool tail = key0 + 32 > S;
        attn_step<NQB, KD, DT>(kf[p], vf[p], qf, mask, m_run, l_run, o, key0, S, n_keys, tail, g, c_exp);
      }
      VVS_ATTN_LOAD(min(step + PD * NW, nsteps - 1), kf[p], vf[p]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#undef VVS_ATTN_LOAD
  VVS_PHASE_MARK(5);
  // merge the partial results of a group's waves: every wave publishes (running maximum, sum, accumulators), then wave aw
  // combines and writes the 16-dim blocks dt = aw, aw + NW, ... for all queries of the group.  The buffers lie where the
  // output tile was: everybody is past the epilogue's reads of it (the barrier in front of the attention).
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = qb * 16 + ql, ui = (ar * 4 + ai) * NQ + qi;
    if (g == 0) { s_m[ui] = m_run[qb]; s_l[ui] = l_run[qb]; }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) s_o[ui * (DH + 1) + dt * 16 + 4 * g + rr] = o[qb][dt][rr];
  }
  __syncthreads();
  VVS_PHASE_MARK(6);
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int qi = qb * 16 + ql, w0 = ar * 4 + qg * NW;   // the group's waves are w0 .. w0 + NW - 1
    float mw[NW], m = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) { mw[w] = s_m[(w0 + w) * NQ + qi]; m = fmaxf(m, mw[w]); }
    const float m_safe = m == -INFINITY ? 0.f : m;
    float wt[NW], l = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {         // fixed order
      wt[w] = exp2f((mw[w] - m_safe) * c_exp);
      l += s_l[(w0 + w) * NQ + qi] * wt[w];
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int dt = aw; dt < DT; dt += NW) {
      float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float* so = s_o + ((w0 + w) * NQ + qi) * (DH + 1) + dt * 16 + 4 * g;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) v[rr] += so[rr] * wt[w];
      }
      if (q0 + qi < T)                     // O-projection operand layout
        *(uint2*)(out + pack_index(r * T + q0 + qi, hd * DH + dt * 16 + 4 * g, d)) =
            make_uint2(pack2bf(v[0] * inv, v[1] * inv), pack2bf(v[2] * inv, v[3] * inv));
    }
  }
  VVS_PHASE_MARK(7);
}

// Tile rows per row of a pair in the fused projection + attention kernel (the padding of its activation operand), or 0
// when a verify call of T block tokens per row does not take that kernel.
int mfma_qkv_attention_rows(const Ctx* c, const PosDesc& pos, int T) {
  if (c->cfg.dtype != VVS_BF16 || c->dh != 64 || T > 64 || !pos.kv_len || !pos.n_emitted || c->d % 64 || c->d / 64 > 64) return 0;
  // 33 .. 64 tokens per row: a workgroup fills a CU (141 KB of LDS), so (head, prompt) pairs beyond the 256 CUs run in rounds,
  // and a poorly filled third round loses to the separate kernels.  Measured at 20 heads, 61 tokens, ms per step fused /
  // separate: 8 prompts 3.99 / 4.30, 12: 4.94 / 5.78, 16: 7.25 / 7.32, 24: 8.73 / 9.02, 28: 10.10 / 9.65, 32: 10.63 / 10.25.
  // (Up to 32 tokens a workgroup is smaller and the fused launch never lost: 13 .. 32 prompts at 27 tokens.)
  if (T > 32 && c->H * c->B > 512) return 0;
  return T <= 32 ? 32 : 64;
}

// q/k/v projection of the row-padded operand A, rotary embedding, cache write and attention in one launch; the result is the
// packed operand of the O projection.
void mfma_qkv_attention(Ctx* c, int layer, const bf16_t* A, const bf16_t* Wqkv, const float* ss, const TreeDesc& tree, const PosDesc& pos,
                        int T, hipStream_t s) {
  GemmEpi ep{};
  set_scale(ep, c, ss);
  ep.kc = (bf16_t*)c->kv + c->kv_layer_stride * layer;
  ep.vc = (bf16_t*)c->kv + c->kv_v_off + c->kv_layer_stride * layer;
  ep.rope = (const float*)(c->ws + c->w.rope_tab);
  ep.T = T; ep.d = c->d; ep.dh = c->dh; ep.S_cap = c->S_cap; ep.rope_pos = c->rope_pos;
  ep.row_stride = c->kv_row_stride; ep.head_stride = c->kv_head_stride;
  ep.pos = pos; ep.tree = tree;
  bf16_t* out = (bf16_t*)(c->ws + c->w.attn);
  const float c_exp = 1.4426950408889634f / sqrtf((float)c->dh);
  constexpr int NSL = 6;                   // 5 stages in flight (TR = 32: 8 slots measured the same, 4 slots 5 % slower)
  dim3 grid(c->H, c->B);
#define VVS_QA(TR, NQB)                                                                                                       \
  {                                                                                                                           \
    constexpr size_t ring = (size_t)NSL * (4 * (TR / 32) + 12) * 1024, tile = (size_t)2 * TR * 196 * sizeof(float);          \
    constexpr size_t lds = (ring > tile ? ring : tile) + (size_t)2 * TR * 72 * sizeof(bf16_t); /* ring / tile / merge, then q */ \
    allow_dynamic_lds(reinterpret_cast<const void*>(&k_qkv_attn<NSL, TR, NQB>), lds);                                         \
    hipLaunchKernelGGL((k_qkv_attn<NSL, TR, NQB>), grid, dim3(512), lds, s, (const uint4*)A, (const uint4*)Wqkv, out, c->d, ep, c_exp); \
  }
  if (T <= 16) VVS_QA(32, 1) else if (T <= 32) VVS_QA(32, 2) else VVS_QA(64, 2)
#undef VVS_QA
}


void mfma_attention(Ctx* c, int layer, const TreeDesc& tree, const PosDesc& pos, int T, hipStream_t s) {
  const bf16_t* q = (const bf16_t*)(c->ws + c->w.q);
  bf16_t* out = (bf16_t*)(c->ws + c->w.attn);
  const bf16_t* kc = (const bf16_t*)c->kv + c->kv_layer_stride * layer;
  const bf16_t* vc = (const bf16_t*)c->kv + c->kv_v_off + c->kv_layer_stride * layer;
  const float c_exp = 1.4426950408889634f / sqrtf((float)c->dh);
  dim3 grid(c->H, c->R);
  const int nqb = T <= 16 ? 1 : (T <= 32 ? 2 : 4);
#define VVS_ATTN(DH, NQB, NW, PD, QG)                                                                                                  \
  hipLaunchKernelGGL((k_attn_mfma<DH, NQB, NW, PD, QG>), grid, dim3(NW * QG * 64), 0, s, q, kc, vc, out, tree, pos, T, c->d, c->kv_row_stride, \
                     c->kv_head_stride, c_exp, c->S_cap >> 5)
  // 4 waves per workgroup keep the register footprint low enough for 2-3 workgroups per CU, so that
  // every (head, row) pair of a call is resident at once
  if (c->dh == 64) {
    if (nqb == 1) VVS_ATTN(64, 1, 4, 2, 1); else if (nqb == 2) VVS_ATTN(64, 2, 4, 2, 1); else VVS_ATTN(64, 2, 2, 2, 2);   // 33 .. 64 queries: two groups of 32
  } else {
    if (nqb == 1) VVS_ATTN(128, 1, 4, 2, 1); else VVS_ATTN(128, 2, 4, 2, 1);   // T <= 32 is enforced at context creation for head size 128
  }
#undef VVS_ATTN
}

}  // namespace vvs
