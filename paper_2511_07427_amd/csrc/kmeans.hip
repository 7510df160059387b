// Prefill: Lloyd's k-means per unit (Section 4.1, Eq. 3-4; Algorithm 1, prefill block; the
// remark of Section 7 that it must cope with empty clusters), cluster statistics, the head-specific
// threshold, and the cluster-contiguous page layout (Section 5.1, intra-cluster placement,
// kept here as the HBM layout).
//
// Every label is the float64 nearest centre (ties to the lowest index): a matrix-core filter in
// float32 settles the clear cases, every point within its error bound is re-assigned by an exact
// float64 scan.  Centre sums are float64 sums over the members.
#include "common.hpp"

namespace dynakv {

namespace {

// One workgroup per unit, first kernel of a build: clears the unit's error word, then flags initial positions
// that are out of range or given twice (the build still runs, with such a position clamped).
__global__ __launch_bounds__(256) void kmeans_check_init_kernel(View v, int N0, const int* init_idx) {
  __shared__ unsigned seen[kMaxPrefill / 32];
  const int u = blockIdx.x, tid = threadIdx.x;
  for (int i = tid; i < kMaxPrefill / 32; i += 256) seen[i] = 0u;
  if (tid == 0) v.err[u] = 0;
  __syncthreads();
  bool bad = false;
  for (int j = tid; j < v.M0; j += 256) {
    const int p = init_idx[(size_t)u * v.M0 + j];
    if (p < 0 || p >= N0) bad = true;
    else if (atomicOr(&seen[p >> 5], 1u << (p & 31)) & (1u << (p & 31))) bad = true;
  }
  if (bad) atomicOr(&v.err[u], DYNAKV_ERR_INIT);
}

// R[u][j] = key at position init_idx[u][j]
__global__ __launch_bounds__(128) void kmeans_init_kernel(View v, const void* X, int N0, const int* init_idx) {
  const int u = blockIdx.y, j = blockIdx.x, d = threadIdx.x;
  int p = init_idx[(size_t)u * v.M0 + j];
  p = min(max(p, 0), N0 - 1);
  unit_R(v, u)[r_index(j, d)] = load_elem(X, ((size_t)u * N0 + p) * kHeadDim + d, v.dtype);
  if (j == 0 && d == 0) { v.xrange[2 * u] = 0x7FFFFFFF; v.xrange[2 * u + 1] = -0x7FFFFFFF; }
}

// ---- order-free centre sums -----------------------------------------------------------------------------
// The centre of a cluster is the float64 sum of its members in ascending position, divided by the count.  Every
// key of a 16-bit type is an integer multiple of 2^q, q = (smallest exponent in the unit) - (mantissa bits), and
// smaller than 2^(emax+1); if (emax + 1 + ceil(log2 N0)) - q <= 53, every partial sum of any subset in any order
// is exactly representable, so the sum does not depend on the order at all and the members need not be sorted
// first: a counting sort that leaves them in arbitrary order is enough.  Units whose keys span too wide a range
// (and float32 keys, and more than 2048 centres) keep the sorted path.
constexpr int kAtomicCentres = 2048;
__global__ __launch_bounds__(256) void kmeans_range_kernel(View v, const void* X, int N0) {
  const int u = blockIdx.y;
  if (v.dtype == DYNAKV_F32) return;
  const uint4* x = (const uint4*)((const uint16_t*)X + (size_t)u * N0 * kHeadDim);
  const int n16 = N0 * kHeadDim / 8;
  const int ebits = v.dtype == DYNAKV_F16 ? 5 : 8, mbits = v.dtype == DYNAKV_F16 ? 10 : 7;
  const int bias = v.dtype == DYNAKV_F16 ? 15 : 127, emask = (1 << ebits) - 1;
  int lo = 0x7FFFFFFF, hi = -0x7FFFFFFF;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n16; i += gridDim.x * 256) {
    const uint4 w = x[i];
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t h = (ww[e >> 1] >> ((e & 1) * 16)) & 0x7FFFu;
      if (h == 0) continue;
      const int eb = (int)(h >> mbits) & emask;
      // subnormals share the grid of the smallest normal exponent; infinities and NaNs make the range unusable
      const int ex = eb == emask ? 0x3FFFFFFF : (eb == 0 ? 1 : eb) - bias;
      lo = min(lo, ex); hi = max(hi, ex);
    }
  }
  for (int o = 32; o > 0; o >>= 1) { lo = min(lo, __shfl_xor(lo, o)); hi = max(hi, __shfl_xor(hi, o)); }
  if ((threadIdx.x & 63) == 0 && hi >= lo) { atomicMin(&v.xrange[2 * u], lo); atomicMax(&v.xrange[2 * u + 1], hi); }
}
// Whether unit u qualifies (see above); q receives the grid exponent.
__device__ inline bool sums_order_free(const View& v, int u, int N0, int* q) {
  if (v.dtype == DYNAKV_F32 || v.M0 > kAtomicCentres) return false;
  const int lo = v.xrange[2 * u], hi = v.xrange[2 * u + 1];
  const int mbits = v.dtype == DYNAKV_F16 ? 10 : 7;
  if (hi < lo) { *q = 0; return true; }               // all keys zero
  int L = 0;
  while ((1 << L) < N0) ++L;
  *q = lo - mbits;
  return hi < 0x3FFFFFFF && (hi + 1 + L) - (lo - mbits) <= 53;
}

// Members of every cluster of the last assignment, in no particular order, for the units whose sums are
// order-free: a counting sort by label (sizes, their prefix, then one LDS counter per cluster hands out the
// places).  One workgroup per unit.  Also the cluster sizes and whether any cluster is empty.
__global__ __launch_bounds__(1024) void kmeans_bucket_kernel(View v, int N0) {
  __shared__ int cnt[kAtomicCentres], off[kAtomicCentres];
  __shared__ int sm[64];
  const int u = blockIdx.x, tid = threadIdx.x;
  int q;
  if (!sums_order_free(v, u, N0, &q)) return;
  for (int j = tid; j < kAtomicCentres; j += 1024) cnt[j] = 0;
  __syncthreads();
  const int* lab = v.labels + (size_t)u * v.Ncap;
  for (int i = tid; i < N0; i += 1024) atomicAdd(&cnt[lab[i]], 1);
  __syncthreads();
  int c2[2], tot = 0, empty = 0;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int j = tid * 2 + k;
    c2[k] = j < v.M0 ? cnt[j] : 0;
    tot += c2[k];
    empty |= j < v.M0 && c2[k] == 0;
  }
  int total;
  int run = block_excl_scan(tot, sm, total);
  int* koff = v.koff + (size_t)u * (v.Mcap + 1);
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int j = tid * 2 + k;
    if (j < v.M0) { off[j] = run; koff[j] = run; v.cn[(size_t)u * v.Mcap + j] = c2[k]; cnt[j] = 0; }
    run += c2[k];
  }
  if (tid == 0) { koff[v.M0] = N0; v.has_empty[u] = 0; }
  __syncthreads();
  if (empty) v.has_empty[u] = 1;
  int* order = v.order + (size_t)u * v.Ncap;
  for (int i = tid; i < N0; i += 1024) {
    const int j = lab[i];
    order[off[j] + atomicAdd(&cnt[j], 1)] = i;
  }
}

// One thread per point: nearest centre in exact float64, centres staged through LDS in tiles.
constexpr int kTileC = 32;
__global__ __launch_bounds__(256) void kmeans_assign_f64_kernel(View v, const void* X, int N0) {
  __shared__ float rs[kTileC][kHeadDim];
  const int u = blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;
  const bool live = i < N0;
  float x[kHeadDim];
  {
    const size_t base = ((size_t)u * N0 + (live ? i : 0)) * kHeadDim;
#pragma unroll
    for (int d8 = 0; d8 < kHeadDim / 8; ++d8) {
      float t[8];
      load8(X, base + d8 * 8, v.dtype, t);
#pragma unroll
      for (int e = 0; e < 8; ++e) x[d8 * 8 + e] = t[e];
    }
  }
  double best = __builtin_inf();
  int arg = 0;
  const float* R = unit_R(v, u);
  for (int j0 = 0; j0 < v.M0; j0 += kTileC) {
    const int nt = min(kTileC, v.M0 - j0);
    __syncthreads();
    for (int t = threadIdx.x; t < nt * kHeadDim; t += 256) rs[t / kHeadDim][t % kHeadDim] = R[r_index(j0 + t / kHeadDim, t % kHeadDim)];
    __syncthreads();
    for (int jj = 0; jj < nt; ++jj) {
      double blk[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        double a = 0.0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const double t = (double)x[k * 8 + e] - (double)rs[jj][k * 8 + e];
          a = fma(t, t, a);
        }
        blk[k] = a;
      }
      double acc = 0.0;
#pragma unroll
      for (int k = 0; k < 16; ++k) acc += blk[k];
      if (acc < best) { best = acc; arg = j0 + jj; }
    }
  }
  if (live) {
    v.labels[(size_t)u * v.Ncap + i] = arg;
    v.dist[(size_t)u * v.Ncap + i] = best;
  }
}

// One workgroup per unit: bitonic sort of (label, position) keys in LDS -> members of every cluster in
// ascending position, and the start of every cluster in that order.
__global__ __launch_bounds__(1024) void kmeans_sort_kernel(View v, int N0, int Npad, int pos_bits, int always) {
  __shared__ uint32_t key[kMaxPrefill];
  const int u = blockIdx.x, tid = threadIdx.x;
  int qx;
  if (!always && sums_order_free(v, u, N0, &qx)) return;       // the order is only needed for the layout
  const int* lab = v.labels + (size_t)u * v.Ncap;
  for (int i = tid; i < Npad; i += 1024) key[i] = i < N0 ? ((uint32_t)lab[i] << pos_bits) | (uint32_t)i : 0xFFFFFFFFu;
  __syncthreads();
  for (int k = 2; k <= Npad; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < Npad; i += 1024) {
        const int ixj = i ^ j;
        if (ixj > i) {
          const uint32_t a = key[i], b = key[ixj];
          const bool up = (i & k) == 0;
          if ((a > b) == up) { key[i] = b; key[ixj] = a; }
        }
      }
      __syncthreads();
    }
  int* order = v.order + (size_t)u * v.Ncap;
  int* koff = v.koff + (size_t)u * (v.Mcap + 1);
  const uint32_t pmask = (1u << pos_bits) - 1;
  if (tid == 0) v.has_empty[u] = 0;
  __syncthreads();
  for (int q = tid; q < N0; q += 1024) {
    const uint32_t kq = key[q];
    order[q] = (int)(kq & pmask);
    const int lq = (int)(kq >> pos_bits);
    const int lp = q ? (int)(key[q - 1] >> pos_bits) : -1;
    for (int l = lp + 1; l <= lq; ++l) koff[l] = q;          // also covers empty clusters in between
    if (lq - lp > 1) v.has_empty[u] = 1;
    if (q == N0 - 1) {
      for (int l = lq + 1; l <= v.M0; ++l) koff[l] = N0;
      if (lq + 1 < v.M0) v.has_empty[u] = 1;
    }
  }
}

// Sixteen lanes per cluster, eight coordinates per lane (one 16-byte load per member of a 16-bit type): centre
// = mean of the members, added one by one in the order of `order` (ascending position after the sort: Eq. 4
// in the fixed order; any order for the units whose sums are order-free).  The 16 lanes fetch the next 16
// member positions with one load while the current 16 rows, all in flight at once, are added.
// grid (ceil(M0/16), U), 256 threads.
template <int DT>
__global__ __launch_bounds__(256) void kmeans_update_kernel(View v, const void* X, int N0) {
  constexpr int RB = DT == DYNAKV_F32 ? 8 : 16;        // rows in flight per lane
  const int u = blockIdx.y, j = blockIdx.x * 16 + (threadIdx.x >> 4), c = threadIdx.x & 15;
  if (j >= v.M0) return;
  const int* koff = v.koff + (size_t)u * (v.Mcap + 1);
  const int* order = v.order + (size_t)u * v.Ncap;
  const int b = koff[j], e = koff[j + 1];
  if (c == 0) v.cn[(size_t)u * v.Mcap + j] = e - b;
  if (e == b) return;
  double s[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) s[k] = 0.0;
  int mine = b + c < e ? order[b + c] : 0;              // lane c holds member c of the current 16
  for (int q0 = b; q0 < e; q0 += 16) {
    const int next = q0 + 16 + c < e ? order[q0 + 16 + c] : 0;
#pragma unroll
    for (int h = 0; h < 16; h += RB) {
      if (q0 + h >= e) break;
      float x[RB][8];
#pragma unroll
      for (int k = 0; k < RB; ++k) {
        const int pos = __shfl(mine, h + k, 16);
        load8(X, ((size_t)u * N0 + pos) * kHeadDim + c * 8, DT, x[k]);
      }
#pragma unroll
      for (int k = 0; k < RB; ++k)
        if (q0 + h + k < e) {
#pragma unroll
          for (int d = 0; d < 8; ++d) s[d] += (double)x[k][d];
        }
    }
    mine = next;
  }
  float* R = unit_R(v, u);
#pragma unroll
  for (int d = 0; d < 8; ++d) R[r_index(j, c * 8 + d)] = (float)(s[d] / (double)(e - b));
}

// One workgroup per unit: every empty cluster, in ascending id, takes the not-yet-taken point that is
// farthest from its own centre (ties to the lowest position).
__global__ __launch_bounds__(256) void kmeans_reseed_kernel(View v, const void* X, int N0) {
  __shared__ double sv[256];
  __shared__ int si[256];
  __shared__ int any_empty;
  const int u = blockIdx.x, tid = threadIdx.x;
  double* dist = v.dist + (size_t)u * v.Ncap;
  if (!v.has_empty[u]) return;
  (void)any_empty;
  for (int j = 0; j < v.M0; ++j) {
    if (v.cn[(size_t)u * v.Mcap + j] != 0) continue;   // uniform across the block
    double bv = -1.0;
    int bi = -1;
    for (int i = tid; i < N0; i += 256) {
      const double t = dist[i];
      if (t > bv) { bv = t; bi = i; }       // ascending i per thread: the first maximum stays
    }
    sv[tid] = bv; si[tid] = bi;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
      if (tid < o) {
        const double ov = sv[tid + o];
        const int oi = si[tid + o];
        if (oi >= 0 && (ov > sv[tid] || (ov == sv[tid] && (si[tid] < 0 || oi < si[tid])))) { sv[tid] = ov; si[tid] = oi; }
      }
      __syncthreads();
    }
    const int far = si[0];
    __syncthreads();
    if (far < 0) break;                      // every point already taken
    if (tid < kHeadDim)
      unit_R(v, u)[r_index(j, tid)] = load_elem(X, ((size_t)u * N0 + far) * kHeadDim + tid, v.dtype);
    if (tid == 0) dist[far] = -2.0;          // taken
    __syncthreads();
  }
}

// ---- assignment through the matrix cores --------------------------------------------------------------
// Filter + exact re-check.  z_ij = <x_i, r_j> - |r_j|^2/2 orders the centres like the squared distance.  The
// filter evaluates it with MFMA on 16-bit operands: x is exact in its storage type, r_j is split into two
// (f16) or three (bf16) 16-bit terms whose sum carries float32 accuracy, accumulation is float32.  The error
// of a filtered z is below eps_i = gamma * |x_i| * max_j |r_j|; a point whose best and second-best filtered
// values are more than 2 eps_i apart has the same nearest centre in exact arithmetic, every other point is
// listed and gets the exact float64 scan (kmeans_exact_kernel), so labels equal the float64 definition.
typedef _Float16 h8v __attribute__((ext_vector_type(8)));
typedef __bf16 b8v __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
// Bound on the relative error of a filtered inner product, |error| <= gamma |x| |r|: the products of two 16-bit
// values are exact in float32; their accumulation (128 per term: 256 for f16's two terms, 384 for bf16's three)
// errs by at most n * 2^-24 of the sum of their magnitudes (2^-16 and 2^-15.4); what the terms leave of r is below
// 2^-22 |r|.  The constants below are twice the sum of those.
constexpr float kFilterGammaF16 = 1.0f / 32768.0f, kFilterGammaBF16 = 1.0f / 16384.0f;

// A-operand order of one 32-cluster tile: [term][k-step of 16][lane][8], lane = (k%16)/8*32 + row.
__device__ inline size_t kmA_index(int nterms, int j, int term, int d) {
  return ((((size_t)(j >> 5) * nterms + term) * 8 + (d >> 4)) * 64 + (((d & 15) >> 3) << 5) + (j & 31)) * 8 + (d & 7);
}

// Thread per centre (lane = centre, so the table reads are contiguous): splits r_j into 16-bit terms in
// A-operand order, stores -|r_j|^2/2 and folds |r_j| into the unit's maximum.  grid (ceil(Mpad/256), U).
__global__ void kmeans_reset_kernel(View v) {
  const int u = blockIdx.x * 256 + threadIdx.x;
  if (u < v.U) { v.rmax[u] = 0.f; v.nflagged[u] = 0; }
}
template <bool BF>
__global__ __launch_bounds__(256) void kmeans_prep_kernel(View v) {
  constexpr int NT = BF ? 3 : 2;
  const int u = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
  const int mpad = (v.M0 + 31) / 32 * 32;
  if (j >= mpad) return;
  const float* R = unit_R(v, u);
  uint16_t* A = v.kmA + (size_t)u * v.kmA_stride;
  double nn = 0.0;
  for (int d8 = 0; d8 < kHeadDim / 8; ++d8) {
    float r[8];
    if (j < v.M0) {
      const f4 a = *(const f4*)(R + r_index(j, d8 * 8)), b = *(const f4*)(R + r_index(j, d8 * 8 + 4));
#pragma unroll
      for (int e = 0; e < 4; ++e) { r[e] = a[e]; r[4 + e] = b[e]; }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = 0.f;
    }
    uint16_t bits[NT][8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      nn += (double)r[e] * (double)r[e];
      float rem = r[e];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        float part;
        if constexpr (BF) { const __bf16 b = (__bf16)rem; part = (float)b; bits[t][e] = __builtin_bit_cast(uint16_t, b); }
        else { const _Float16 hh = (_Float16)rem; part = (float)hh; bits[t][e] = __builtin_bit_cast(uint16_t, hh); }
        rem -= part;
      }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      uint4 w;
      w.x = bits[t][0] | ((uint32_t)bits[t][1] << 16); w.y = bits[t][2] | ((uint32_t)bits[t][3] << 16);
      w.z = bits[t][4] | ((uint32_t)bits[t][5] << 16); w.w = bits[t][6] | ((uint32_t)bits[t][7] << 16);
      *(uint4*)(A + kmA_index(NT, j, t, d8 * 8)) = w;
    }
  }
  v.hn[(size_t)u * mpad + j] = j < v.M0 ? (float)(-0.5 * nn) : -__builtin_inff();
  if (j < v.M0) atomicMax((int*)&v.rmax[u], __float_as_int((float)sqrt(nn) * 1.000001f));   // non-negative floats order like ints
}

// grid (ceil(N0/256), U); 4 wavefronts x 64 points.  Z^T = R~ X^T in 32x32 tiles: lane (p, h) ends up with the
// filtered values of point p for the centres 8*(i/4) + 4*h + i%4 of every tile, so the running best / second
// best need no cross-lane work until the very end.
template <bool BF>
__global__ __launch_bounds__(256, 3) void kmeans_assign_mfma_kernel(View v, const void* X, int N0) {
  constexpr int NT = BF ? 3 : 2;
  __shared__ uint4 sA[2][NT * 8 * 64];     // two tiles: the next one is fetched while this one is consumed
  __shared__ float shn[2][32];
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int p = lane & 31, h = lane >> 5;
  const int ntiles = (v.M0 + 31) / 32;
  const int pbase = blockIdx.x * 256 + wave * 64;
  uint4 bx[2][8];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int pt = pbase + t * 32 + p;
    const uint16_t* xr = (const uint16_t*)X + ((size_t)u * N0 + (pt < N0 ? pt : 0)) * kHeadDim + h * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) bx[t][ks] = pt < N0 ? *(const uint4*)(xr + ks * 16) : uint4{0, 0, 0, 0};
  }
  float xnorm[2];                               // |x| of this lane's point, from the operand registers
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    float nn = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uint32_t ww[4] = {bx[t][ks].x, bx[t][ks].y, bx[t][ks].z, bx[t][ks].w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint16_t hh = (uint16_t)(ww[e >> 1] >> ((e & 1) * 16));
        const float x = BF ? bf16_to_float(hh) : f16_to_float(hh);
        nn += x * x;
      }
    }
    nn += __shfl_xor(nn, 32);
    xnorm[t] = __builtin_sqrtf(nn) * 1.0001f;
  }
  float best[2] = {-__builtin_inff(), -__builtin_inff()}, second[2] = {-__builtin_inff(), -__builtin_inff()};
  int bidx[2] = {0, 0};
  const uint4* gA = (const uint4*)(v.kmA + (size_t)u * v.kmA_stride);
  const float* hn = v.hn + (size_t)u * ntiles * 32;
  // Tiles travel global -> registers -> LDS one iteration ahead of their use (plain scalars, so that they stay
  // in registers); the empty asm statement keeps the compiler from sinking the loads down to the LDS stores.
  uint4 st0, st1, st2, st3, st4 = {0, 0, 0, 0}, st5 = {0, 0, 0, 0};
  float sh = 0.f;
#define KM_FETCH(tile)                                                        \
  {                                                                           \
    const uint4* g_ = gA + (size_t)(tile) * NT * 512 + tid;                   \
    st0 = g_[0]; st1 = g_[256]; st2 = g_[512]; st3 = g_[768];                 \
    if constexpr (NT == 3) { st4 = g_[1024]; st5 = g_[1280]; }                \
    if (tid < 32) sh = hn[(tile) * 32 + tid];                                 \
    asm volatile("" ::: "memory");                                            \
  }
#define KM_COMMIT(buf)                                                        \
  {                                                                           \
    uint4* d_ = sA[buf] + tid;                                                \
    d_[0] = st0; d_[256] = st1; d_[512] = st2; d_[768] = st3;                 \
    if constexpr (NT == 3) { d_[1024] = st4; d_[1280] = st5; }                \
    if (tid < 32) shn[buf][tid] = sh;                                         \
  }
  KM_FETCH(0);
  KM_COMMIT(0);
  __syncthreads();
  for (int tile = 0; tile < ntiles; ++tile) {
    const int cur = tile & 1;
    if (tile + 1 < ntiles) KM_FETCH(tile + 1);
    f16v acc[2];
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[0][i] = shn[cur][8 * (i >> 2) + 4 * h + (i & 3)]; acc[1][i] = acc[0][i]; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int term = 0; term < NT; ++term) {
        const uint4 a = sA[cur][(term * 8 + ks) * 64 + lane];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          if constexpr (BF)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(b8v, a), __builtin_bit_cast(b8v, bx[t][ks]), acc[t], 0, 0, 0);
          else
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8v, a), __builtin_bit_cast(h8v, bx[t][ks]), acc[t], 0, 0, 0);
        }
      }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float val = acc[t][i];
        second[t] = __builtin_amdgcn_fmed3f(best[t], second[t], val);      // second <= best: the median is the runner-up
        if (val > best[t]) bidx[t] = tile * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
        best[t] = fmaxf(best[t], val);
      }
    if (tile + 1 < ntiles) KM_COMMIT(cur ^ 1);
    __syncthreads();
  }
#undef KM_FETCH
#undef KM_COMMIT
  const float rmax = v.rmax[u];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const float ob = __shfl_xor(best[t], 32), os = __shfl_xor(second[t], 32);
    const int oi = __shfl_xor(bidx[t], 32);
    const float nb = fmaxf(best[t], ob), ns = fmaxf(fmaxf(second[t], os), fminf(best[t], ob));
    const int idx = (ob > best[t] || (ob == best[t] && oi < bidx[t])) ? oi : bidx[t];
    const int pt = pbase + t * 32 + p;
    if (h == 0 && pt < N0) {
      v.labels[(size_t)u * v.Ncap + pt] = idx;
      const float eps = (BF ? kFilterGammaBF16 : kFilterGammaF16) * xnorm[t] * rmax + 2.4e-7f * rmax * rmax;
      if (!(nb - ns > 2.f * eps)) v.order[(size_t)u * v.Ncap + atomicAdd(&v.nflagged[u], 1)] = pt;
    }
  }
}

// Exact nearest centre (float64, left to right, ties to the lowest id) of every listed point: one workgroup
// per point, thread = centre, so the centroid table is read 1 KB per wavefront at a time.  grid (B, U).
__global__ __launch_bounds__(256) void kmeans_exact_kernel(View v, const void* X, int N0) {
  __shared__ double xd[kHeadDim];
  __shared__ double sv[256];
  __shared__ int si[256];
  const int u = blockIdx.y, tid = threadIdx.x;
  const int nf = v.nflagged[u];
  const float* R = unit_R(v, u);
  for (int f = blockIdx.x; f < nf; f += gridDim.x) {
    const int pt = v.order[(size_t)u * v.Ncap + f];
    __syncthreads();
    if (tid < kHeadDim) xd[tid] = (double)load_elem(X, ((size_t)u * N0 + pt) * kHeadDim + tid, v.dtype);
    __syncthreads();
    double best = __builtin_inf();
    int arg = -1;
    for (int j = tid; j < v.M0; j += 256) {
      f4 row[8];
      load_centroid_head(R, j, row);
      double dist[1];
      centroid_sums<1>(R, j, row, dist, [&](int d, float rv, double (&a)[1]) __attribute__((always_inline)) {
        const double t = xd[d] - (double)rv;
        a[0] = fma(t, t, a[0]);
      });
      const double acc = dist[0];
      if (acc < best || arg < 0) { best = acc; arg = j; }
    }
    block_arg_reduce<false>(best, arg, sv, si);
    if (tid == 0) v.labels[(size_t)u * v.Ncap + pt] = si[0];
  }
}

// Only when some cluster came out empty: the distance of every point to the centre it was assigned to (the
// centres of this assignment, i.e. before the update), which the re-seeding step ranks.
__global__ __launch_bounds__(256) void kmeans_dist_kernel(View v, const void* X, int N0) {
  const int u = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
  if (!v.has_empty[u] || i >= N0) return;
  const int j = v.labels[(size_t)u * v.Ncap + i];
  const float* R = unit_R(v, u);
  const size_t base = ((size_t)u * N0 + i) * kHeadDim;
  v.dist[(size_t)u * v.Ncap + i] = blocked16([&](int k) __attribute__((always_inline)) {
    float x[8];
    load8(X, base + k * 8, v.dtype, x);
    const f4 ra = *(const f4*)(R + r_index(j, k * 8)), rb = *(const f4*)(R + r_index(j, k * 8 + 4));
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const double t = (double)x[e] - (double)(e < 4 ? ra[e] : rb[e - 4]);
      acc = fma(t, t, acc);
    }
    return acc;
  });
}

// dist[i] = squared distance of point i to the (updated) centre of its own cluster.  Sixteen lanes per point, one
// block of 8 coordinates each; the 16 block sums are then added left to right by one thread per point.  Points
// are taken in the sorted order (by cluster), so the 16 points of a workgroup mostly share one centre and its
// lines of the lane-interleaved table are fetched once.
__global__ __launch_bounds__(256) void point_dist_kernel(View v, const void* X, int N0) {
  __shared__ double bs[16][17];
  const int u = blockIdx.y, p = threadIdx.x >> 4, k = threadIdx.x & 15;
  const int i = v.order[(size_t)u * v.Ncap + min((int)blockIdx.x * 16 + p, N0 - 1)];
  const int j = v.labels[(size_t)u * v.Ncap + i];
  const float* R = unit_R(v, u);
  float x[8];
  load8(X, ((size_t)u * N0 + i) * kHeadDim + k * 8, v.dtype, x);
  const f4 ra = *(const f4*)(R + r_index(j, k * 8)), rb = *(const f4*)(R + r_index(j, k * 8 + 4));
  double acc = 0.0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const double t = (double)x[e] - (double)(e < 4 ? ra[e] : rb[e - 4]);
    acc = fma(t, t, acc);
  }
  bs[p][k] = acc;
  __syncthreads();
  // (thread 16 t holds the index of point t of the workgroup)
  if ((threadIdx.x & 15) == 0 && blockIdx.x * 16 + p < N0)
    v.dist[(size_t)u * v.Ncap + i] = blocked16([&](int kk) __attribute__((always_inline)) { return bs[p][kk]; });
}

// One workgroup per unit: per-cluster n, M2 (members in order), page chains, tau, counters.
__global__ __launch_bounds__(1024) void finalize_kernel(View v, int N0) {
  __shared__ int sm[64];
  __shared__ double jsum[16];                   // per-wavefront sums of M2, for the objective that gives tau
  static_assert(kMaxInitClusters <= 8 * 1024, "eight consecutive clusters per thread cover every initial cluster");
  const int u = blockIdx.x, tid = threadIdx.x;
  const int* koff = v.koff + (size_t)u * (v.Mcap + 1);
  const int* order = v.order + (size_t)u * v.Ncap;
  const double* dist = v.dist + (size_t)u * v.Ncap;
  const size_t cb = (size_t)u * v.Mcap;
  // pages per cluster, 8 consecutive clusters per thread
  int np[8], tot = 0;
  for (int k = 0; k < 8; ++k) {
    const int j = tid * 8 + k;
    np[k] = j < v.M0 ? (koff[j + 1] - koff[j] + kPageTokens - 1) / kPageTokens : 0;
    tot += np[k];
  }
  int total;
  int base = block_excl_scan(tot, sm, total);
  for (int k = 0; k < 8; ++k) {
    const int j = tid * 8 + k;
    if (j >= v.Mcap) break;
    if (j < v.M0) {
      v.cn[cb + j] = koff[j + 1] - koff[j];
      v.csz[cb + j] = koff[j + 1] - koff[j];
      v.pg_off[cb + j] = base;
      for (int p = 0; p < kInlinePages; ++p) v.cpg[(cb + j) * kInlinePages + p] = p < np[k] ? base + p : -1;
      v.ctail[cb + j] = np[k] ? base + np[k] - 1 : -1;
      for (int p = 0; p < np[k]; ++p) v.pnext[(size_t)u * v.Pcap + base + p] = p + 1 < np[k] ? base + p + 1 : -1;
      base += np[k];
    } else {
      v.cn[cb + j] = 0; v.csz[cb + j] = 0; v.cM2[cb + j] = 0.0; v.ctail[cb + j] = -1;
      for (int p = 0; p < kInlinePages; ++p) v.cpg[(cb + j) * kInlinePages + p] = -1;
    }
    v.cb[cb + j] = 0; v.cflag[cb + j] = 0; v.in_req[cb + j] = 0; v.score[cb + j] = 0.f;
  }
  for (int j = 8 * 1024 + tid; j < v.Mcap; j += 1024) {          // slots that no thread's run of eight reaches
    v.cn[cb + j] = 0; v.csz[cb + j] = 0; v.cM2[cb + j] = 0.0; v.ctail[cb + j] = -1;
    for (int p = 0; p < kInlinePages; ++p) v.cpg[(cb + j) * kInlinePages + p] = -1;
    v.cb[cb + j] = 0; v.cflag[cb + j] = 0; v.in_req[cb + j] = 0; v.score[cb + j] = 0.f;
  }
  // M2 of cluster j = sum of its members' distances in storage order: one thread per cluster, eight members
  // requested at a time, added one by one
  double jmine = 0.0;
  for (int j = tid; j < v.M0; j += 1024) {
    const int b = koff[j], e = koff[j + 1];
    double m2 = 0.0;
    for (int q0 = b; q0 < e; q0 += 8) {
      int o[8];
      double x[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) o[k] = order[min(q0 + k, e - 1)];
#pragma unroll
      for (int k = 0; k < 8; ++k) x[k] = dist[o[k]];
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (q0 + k < e) m2 += x[k];
    }
    v.cM2[cb + j] = m2;
    jmine += m2;
  }
  for (int o = 32; o > 0; o >>= 1) jmine += __shfl_xor(jmine, o);
  if ((tid & 63) == 0) jsum[tid >> 6] = jmine;
  if (v.dtype != DYNAKV_F32) {               // search copy of the final centroids
    const float* R = unit_R(v, u);
    uint16_t* Rq = unit_Rq(v, u);
    for (int t = tid; t < v.M0 * kHeadDim; t += 1024)
      Rq[rq_index(t >> 7, t & 127)] = round_bits16(R[r_index(t >> 7, t & 127)], v.dtype);
  }
  __syncthreads();
  if (tid == 0) {
    double J = 0.0;
    for (int w = 0; w < 16; ++w) J += jsum[w];
    v.tau[u] = (double)v.var_alpha * (J / (double)N0);
    v.M[u] = v.M0; v.N[u] = N0; v.nflag[u] = 0; v.n_sel[u] = 0; v.t_sel[u] = 0; v.n_list[u] = 0;
    v.ticket[u] = 0; v.bump[u] = total; v.free_top[u] = 0; v.last_assign[u] = -1; v.lcount[u] = 0; v.rmax2[u] = 0;
    for (int k = 0; k < kCounters; ++k) v.counters[(size_t)u * kCounters + k] = 0;
  }
}

// 16 consecutive entries of the sorted order per workgroup, 16 threads per entry, 8 coordinates per thread:
// keys and values move as whole 16-byte chunks of their token's rows.
__global__ __launch_bounds__(256) void layout_copy_kernel(View v, const void* K, const void* V, int N0) {
  const int u = blockIdx.y, q = blockIdx.x * 16 + (threadIdx.x >> 4), c = threadIdx.x & 15;
  if (q >= N0) return;
  const int pos = v.order[(size_t)u * v.Ncap + q];
  const int j = v.labels[(size_t)u * v.Ncap + pos];
  const int rank = q - v.koff[(size_t)u * (v.Mcap + 1) + j];
  const int page = v.pg_off[(size_t)u * v.Mcap + j] + rank / kPageTokens, slot = rank % kPageTokens;
  char* pg = page_ptr(v, u, page);
  const size_t src = ((size_t)u * N0 + pos) * kHeadDim + c * 8;
  if (v.dtype == DYNAKV_F32) {
    const f4* ks = (const f4*)((const float*)K + src);
    const f4* vs = (const f4*)((const float*)V + src);
    *(f4*)((float*)pg + k_index32(slot, c * 8)) = ks[0];
    *(f4*)((float*)pg + k_index32(slot, c * 8 + 4)) = ks[1];
    *(f4*)((float*)pg + v_index32(slot, c * 8)) = vs[0];
    *(f4*)((float*)pg + v_index32(slot, c * 8 + 4)) = vs[1];
  } else {
    *(uint4*)((uint16_t*)pg + k_index16(slot, c * 8)) = *(const uint4*)((const uint16_t*)K + src);
    *(uint4*)((uint16_t*)pg + v_index16(slot, c * 8)) = *(const uint4*)((const uint16_t*)V + src);
  }
  if (c == 0) v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + slot] = pos;
}

}  // namespace

hipError_t launch_build_index(const View& v, const void* K, const void* V, int N0, const int* init_idx, int iters,
                              void* ws, size_t ws_bytes, hipStream_t st) {
  (void)ws; (void)ws_bytes;
  kmeans_check_init_kernel<<<v.U, 256, 0, st>>>(v, N0, init_idx);
  kmeans_init_kernel<<<dim3(v.M0, v.U), 128, 0, st>>>(v, K, N0, init_idx);
  kmeans_range_kernel<<<dim3(16, v.U), 256, 0, st>>>(v, K, N0);
  int Npad = 2, pos_bits = 1;
  while (Npad < N0) { Npad <<= 1; ++pos_bits; }
  const dim3 gpts((N0 + 255) / 256, v.U);
  const bool mfma = v.dtype != DYNAKV_F32;     // float32 keys keep the plain float64 scan
  const bool atomic_path = mfma && v.M0 <= kAtomicCentres;   // per unit, the kernels decide by the keys' range
  const dim3 gprep(((v.M0 + 31) / 32 * 32 + 255) / 256, v.U);
  for (int it = 0; it < iters; ++it) {
    if (mfma) {
      if (v.dtype == DYNAKV_F16) {
        kmeans_reset_kernel<<<(v.U + 255) / 256, 256, 0, st>>>(v);
        kmeans_prep_kernel<false><<<gprep, 256, 0, st>>>(v);
        kmeans_assign_mfma_kernel<false><<<gpts, 256, 0, st>>>(v, K, N0);
      } else {
        kmeans_reset_kernel<<<(v.U + 255) / 256, 256, 0, st>>>(v);
        kmeans_prep_kernel<true><<<gprep, 256, 0, st>>>(v);
        kmeans_assign_mfma_kernel<true><<<gpts, 256, 0, st>>>(v, K, N0);
      }
      kmeans_exact_kernel<<<dim3(64, v.U), 256, 0, st>>>(v, K, N0);
    } else {
      kmeans_assign_f64_kernel<<<gpts, 256, 0, st>>>(v, K, N0);
    }
    kmeans_sort_kernel<<<v.U, 1024, 0, st>>>(v, N0, Npad, pos_bits, it + 1 == iters);
    if (atomic_path && it + 1 < iters) kmeans_bucket_kernel<<<v.U, 1024, 0, st>>>(v, N0);
    if (it + 1 < iters) kmeans_dist_kernel<<<gpts, 256, 0, st>>>(v, K, N0);
    const dim3 gupd((v.M0 + 15) / 16, v.U);
    if (v.dtype == DYNAKV_F32) kmeans_update_kernel<DYNAKV_F32><<<gupd, 256, 0, st>>>(v, K, N0);
    else if (v.dtype == DYNAKV_F16) kmeans_update_kernel<DYNAKV_F16><<<gupd, 256, 0, st>>>(v, K, N0);
    else kmeans_update_kernel<DYNAKV_BF16><<<gupd, 256, 0, st>>>(v, K, N0);
    if (it + 1 < iters) kmeans_reseed_kernel<<<v.U, 256, 0, st>>>(v, K, N0);
  }
  point_dist_kernel<<<dim3((N0 + 15) / 16, v.U), 256, 0, st>>>(v, K, N0);
  finalize_kernel<<<v.U, 1024, 0, st>>>(v, N0);
  layout_copy_kernel<<<dim3((N0 + 15) / 16, v.U), 256, 0, st>>>(v, K, V, N0);
  return hipGetLastError();
}

}  // namespace dynakv
