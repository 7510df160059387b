// Query x centroid scores and the distances of a new entry on the matrix cores (Section 4.1: similarity between
// the query and every representative; Algorithm 1, decode block: nearest cluster of the new entry), over the
// 16-bit search copy of the centroids, and the float64 evaluations that retake every decision which the float32
// accumulation could change.
//
// One contraction does both: rows = the G query heads and (in a step that appends) the new key, columns = the 16
// clusters of a tile, 128 coordinates in four v_mfma_f32_16x16x32 instructions.  Products of two 16-bit values are
// exact in float32; only the accumulation rounds: |error| <= 128 * 2^-24 * |row| |centroid| (the bounds below
// use that, with 1 % on top for the float32 norms).  |centroid|^2 comes from the same operand multiplied by itself (diagonal of the tile's Gram
// matrix).
#pragma once
#include "append.hpp"

namespace dynakv {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));

constexpr float kAccBound = 1.0f / 131072.0f;     // 128 * 2^-24: float32 accumulation of 128 exact products, standard model

template <bool BF>
__device__ __forceinline__ f4 mfma_k32(const uint4& a, const uint4& b, f4 c) {
  if constexpr (BF)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
}

__device__ __forceinline__ float sel4(const f4& a, int i) { return i == 0 ? a[0] : i == 1 ? a[1] : i == 2 ? a[2] : a[3]; }

// Rows of the contraction as A operands: lane l holds coordinates 32 s + 8 (l / 16) .. + 7 of row 16 blk + l % 16.
// Row r < G is query head r of unit u, row G the new key (kin != null), the others are zero.
template <int NBLK>
struct ScoreRows {
  uint4 a[NBLK][4];
};
template <int NBLK>
__device__ inline void load_score_rows(ScoreRows<NBLK>& A, int G, const void* Q, const void* kin, int u, int lane) {
  const int lg = lane >> 4;
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk) {
    const int r = (lane & 15) + 16 * blk;
    const uint16_t* p = r < G ? (const uint16_t*)Q + ((size_t)u * G + r) * kHeadDim
                              : (r == G && kin) ? (const uint16_t*)kin + (size_t)u * kHeadDim : nullptr;
#pragma unroll
    for (int s = 0; s < 4; ++s) A.a[blk][s] = p ? *(const uint4*)(p + 32 * s + 8 * lg) : uint4{0, 0, 0, 0};
  }
}

// Norms of the rows, for the error bounds: qbound = max_g |q_g| (group max) or sum_g |q_g| (group sum), kn = |new key|.
struct RowNorms {
  float qbound, kn;
};
template <bool BF, int NBLK>
__device__ inline RowNorms row_norms(const ScoreRows<NBLK>& A, int G, int group_reduce, int lane) {
  RowNorms n{0.f, 0.f};
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk) {
    float s2 = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint32_t ww[4] = {A.a[blk][s].x, A.a[blk][s].y, A.a[blk][s].z, A.a[blk][s].w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint16_t h = (uint16_t)(ww[e >> 1] >> ((e & 1) * 16));
        const float x = BF ? bf16_to_float(h) : f16_to_float(h);
        s2 = fmaf(x, x, s2);
      }
    }
    s2 += __shfl_xor(s2, 16);
    s2 += __shfl_xor(s2, 32);
    const int r = (lane & 15) + 16 * blk;
    const float nr = __builtin_sqrtf(s2) * 1.0001f;
    float q = r < G ? nr : 0.f, k = r == G ? nr : 0.f;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const float oq = __shfl_xor(q, o);
      q = group_reduce == DYNAKV_GROUP_MAX ? fmaxf(q, oq) : q + oq;
      k = fmaxf(k, __shfl_xor(k, o));
    }
    n.qbound = group_reduce == DYNAKV_GROUP_MAX ? fmaxf(n.qbound, q) : n.qbound + q;
    n.kn = fmaxf(n.kn, k);
  }
  return n;
}

// One tile: b[s] = this lane's 16 bytes of chunk s.  Returns in EVERY lane, for cluster lane % 16 of the tile:
//   red   the group-reduced inner product over the query heads (before the softmax scale)
//   kdot  <new key, centroid>            (NEAR)
//   nrm2  |centroid|^2
template <bool BF, int NBLK, bool NEAR>
__device__ __forceinline__ void score_tile(const uint4 (&b)[4], const ScoreRows<NBLK>& A, int G, int group_reduce, int lane,
                                           float& red, float& kdot, float& nrm2) {
  const int lg = lane >> 4;
  f4 acc[NBLK], gram = {0, 0, 0, 0};
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk) {
    acc[blk] = f4{0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 4; ++s) acc[blk] = mfma_k32<BF>(A.a[blk][s], b[s], acc[blk]);
  }
#pragma unroll
  for (int s = 0; s < 4; ++s) gram = mfma_k32<BF>(b[s], b[s], gram);
  // acc[blk][i] = <row 16 blk + 4 lg + i, cluster lane % 16>
  const bool mx = group_reduce == DYNAKV_GROUP_MAX;
  red = mx ? -__builtin_inff() : 0.f;
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (16 * blk + 4 * lg + i < G) red = mx ? fmaxf(red, acc[blk][i]) : red + acc[blk][i];
  if (G > 4) {
    const float o = __shfl_xor(red, 16);
    red = mx ? fmaxf(red, o) : red + o;
  }
  if (G > 8) {
    const float o = __shfl_xor(red, 32);
    red = mx ? fmaxf(red, o) : red + o;
  }
  if constexpr (NEAR) {      // row G sits in lane group (G % 16) / 4, register G % 4 of block G / 16
    const float mine = NBLK == 2 && G >= 16 ? sel4(acc[NBLK - 1], G & 3) : sel4(acc[0], G & 3);
    kdot = __shfl(mine, (lane & 15) + 16 * ((G & 15) >> 2));
  } else {
    kdot = 0.f;
  }
  // gram[i] = <cluster 4 lg + i, cluster lane % 16>: the diagonal entry of cluster c sits in lane c + 16 (c / 4),
  // register c % 4
  const int c = lane & 15;
  nrm2 = __shfl(sel4(gram, c & 3), c + 16 * (c >> 2));
}

// ---- float64 evaluations on the search copy (16-bit) -----------------------------------------------------
// Squared distance of the key kd[0..127] (float64, LDS) to the search copy of cluster j, one thread.
__device__ inline double exact_sqdist16(const uint16_t* Rq, int j, const double* kd, int dtype) {
  double acc = 0.0;
#pragma unroll 2
  for (int d8 = 0; d8 < kHeadDim / 8; ++d8) {
    float x[8];
    load8(Rq, rq_index(j, d8 * 8), dtype, x);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const double t = kd[d8 * 8 + e] - (double)x[e];
      acc = fma(t, t, acc);
    }
  }
  return acc;
}

// Score of cluster j in float64, by the four lanes of a quad (lane q of it takes coordinates 32 q .. 32 q + 31);
// every lane of the quad gets the result: scale * reduce_g <q_g, r~_j>, rounded to float32 if the index says so.
__device__ inline double quad_exact_score(const View& v, const uint16_t* Rq, const void* Q, int u, int j, int q) {
  float r[32];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float x[8];
    load8(Rq, rq_index(j, 32 * q + 8 * k), v.dtype, x);
#pragma unroll
    for (int e = 0; e < 8; ++e) r[8 * k + e] = x[e];
  }
  double red = 0.0;
  for (int g = 0; g < v.G; ++g) {
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float x[8];
      load8(Q, ((size_t)u * v.G + g) * kHeadDim + 32 * q + 8 * k, v.dtype, x);
#pragma unroll
      for (int e = 0; e < 8; ++e) s = fma((double)x[e], (double)r[8 * k + e], s);
    }
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    red = g == 0 ? s : v.group_reduce == DYNAKV_GROUP_MAX ? fmax(red, s) : red + s;
  }
  const double e = red * v.scale_d;
  return v.score_round ? (double)(float)e : e;
}

// ---- nearest cluster of the new key ----------------------------------------------------------------------
// (zb, jb, z2) = largest value, its index (lowest among equals; < 0: none) and the second largest value of a set;
// merges the triple of a disjoint set into it.
__device__ __forceinline__ void merge_best2(float& zb, int& jb, float& z2, float ob, int oj, float o2) {
  const bool take = oj >= 0 && (jb < 0 || ob > zb || (ob == zb && oj < jb));
  const float loser = take ? zb : ob;                   // the better of the two bests stays, the other competes for second
  const bool loser_ok = take ? jb >= 0 : oj >= 0;
  if (take) { zb = ob; jb = oj; }
  z2 = fmaxf(fmaxf(z2, o2), loser_ok ? loser : -__builtin_inff());
}
// The same over the 64 lanes of a wavefront; every lane gets the result.  Butterfly inside each row of 16 lanes
// (the sets that meet are disjoint at every step), then row to row, then the last lane's triple for everybody.
template <int CTRL, int ROWS>
__device__ __forceinline__ void best2_step(float& zb, int& jb, float& z2) {
  // a lane that gets nothing from this step (its row is masked out) merges the empty set: index -1, -inf
  const float ob = __int_as_float(dpp_or<CTRL, ROWS>(0, __float_as_int(zb)));
  const int oj = dpp_or<CTRL, ROWS>(-1, jb);
  const float o2 = __int_as_float(dpp_or<CTRL, ROWS>(__float_as_int(-__builtin_inff()), __float_as_int(z2)));
  merge_best2(zb, jb, z2, ob, oj, o2);
}
__device__ __forceinline__ void wave_best2(float& zb, int& jb, float& z2) {
  best2_step<kDppXor1, 0xF>(zb, jb, z2);
  best2_step<kDppXor2, 0xF>(zb, jb, z2);
  best2_step<kDppHalfMirror, 0xF>(zb, jb, z2);
  best2_step<kDppMirror, 0xF>(zb, jb, z2);
  best2_step<kDppBcast15, 0xA>(zb, jb, z2);
  best2_step<kDppBcast31, 0xC>(zb, jb, z2);
  zb = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(zb), 63));
  jb = __builtin_amdgcn_readlane(jb, 63);
  z2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(z2), 63));
}

// Every thread brings the best and the second best z it has seen (z_j = <k, r~_j> - |r~_j|^2 / 2 as the matrix
// cores computed it: largest = nearest; jb < 0: none) and the whole workgroup of NT threads gets the cluster that
// exact arithmetic finds nearest (lowest id among equals): if the runner-up lies beyond the error bound of the
// best, the best is it; otherwise every cluster within the bound (read back from zd[0..M), which the caller has
// made visible to the workgroup) is evaluated in float64.  kd: the key in float64 (LDS); kn, rmax2: |k| and the
// largest |r~_j|^2.  sv / si / s2: 16 entries of LDS each.
// Second half of nearest_resolve: every wavefront's (best, its cluster, runner-up) is in sv / si / s2 [0 .. NT / 64)
// and a barrier lies behind that.
template <int NT>
__device__ inline int nearest_decide(const View& v, int u, int M, float kn, float rmax2, const float* zd, const uint16_t* Rq,
                                     const double* kd, double* sv, int* si, float* s2) {
  float zb = (float)sv[0], z2 = s2[0];
  int jb = si[0];
#pragma unroll
  for (int k = 1; k < NT / 64; ++k) merge_best2(zb, jb, z2, (float)sv[k], si[k], s2[k]);
  const float rmax = __builtin_sqrtf(rmax2) * 1.0001f;
  const float eps = kAccBound * (kn * rmax + 0.5f * rmax * rmax) * 1.01f;
  if (jb < 0 || zb - z2 > 2.f * eps) return jb;        // workgroup-uniform
  // several clusters within the bound of the best: float64 distances of all of them (read back from memory)
  __syncthreads();
  const float thr = zb - 2.f * eps;
  double best = __builtin_inf();
  int arg = -1;
  for (int j = threadIdx.x; j < M; j += NT)
    if (zd[j] >= thr) {
      const double dj = exact_sqdist16(Rq, j, kd, v.dtype);
      if (arg < 0 || dj < best) { best = dj; arg = j; }
    }
  if (threadIdx.x == 0) count(v, u, 7, 1);
  return block_argmin<NT>(best, arg, sv, si);
}
template <int NT>
__device__ inline int nearest_resolve(const View& v, int u, int M, float zb, int jb, float z2, float kn, float rmax2,
                                      const float* zd, const uint16_t* Rq, const double* kd, double* sv, int* si,
                                      float* s2) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  wave_best2(zb, jb, z2);
  lds_barrier();
  if (lane == 0) { sv[w] = (double)zb; si[w] = jb; s2[w] = z2; }
  lds_barrier();
  return nearest_decide<NT>(v, u, M, kn, rmax2, zd, Rq, kd, sv, si, s2);
}

}  // namespace dynakv
