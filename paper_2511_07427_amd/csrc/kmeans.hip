// Prefill: Lloyd's k-means per unit (Section 4.1, Eq. 3-4; Algorithm 1, prefill block; the
// "robust to empty clusters" remark of Section 7), cluster statistics, the head-specific
// threshold, and the cluster-contiguous page layout (Section 5.1, intra-cluster placement,
// kept here as the HBM layout).
//
// Every decision is taken on float64 squared distances accumulated left to right over the
// coordinate index, ties to the lowest index; centroid sums run over members in ascending
// position, so the result does not depend on how the work is spread over the machine.
#include "common.hpp"

namespace dynakv {

namespace {

__global__ void fill32_kernel(uint32_t* p, size_t n, uint32_t val) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = val;
}

// R[u][j] = key at position init_idx[u][j]
__global__ __launch_bounds__(128) void kmeans_init_kernel(View v, const void* X, int N0, const int* init_idx) {
  const int u = blockIdx.y, j = blockIdx.x, d = threadIdx.x;
  int p = init_idx[(size_t)u * v.M0 + j];
  p = min(max(p, 0), N0 - 1);
  unit_R(v, u)[r_index(j, d)] = load_elem(X, ((size_t)u * N0 + p) * kHeadDim + d, v.dtype);
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
    for (int d = 0; d < kHeadDim; ++d) x[d] = load_elem(X, base + d, v.dtype);
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
      double acc = 0.0;
#pragma unroll
      for (int d = 0; d < kHeadDim; ++d) {
        const double t = (double)x[d] - (double)rs[jj][d];
        acc = fma(t, t, acc);
      }
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
__global__ __launch_bounds__(1024) void kmeans_sort_kernel(View v, int N0, int Npad, int pos_bits) {
  __shared__ uint32_t key[kMaxPrefill];
  const int u = blockIdx.x, tid = threadIdx.x;
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
  for (int q = tid; q < N0; q += 1024) {
    const uint32_t kq = key[q];
    order[q] = (int)(kq & pmask);
    const int lq = (int)(kq >> pos_bits);
    const int lp = q ? (int)(key[q - 1] >> pos_bits) : -1;
    for (int l = lp + 1; l <= lq; ++l) koff[l] = q;          // also covers empty clusters in between
    if (q == N0 - 1)
      for (int l = lq + 1; l <= v.M0; ++l) koff[l] = N0;
  }
}

// Thread (cluster, coordinate): centre = mean of the members, summed in ascending position (Eq. 4).
__global__ __launch_bounds__(256) void kmeans_update_kernel(View v, const void* X, int N0) {
  const int u = blockIdx.y, j = blockIdx.x * 2 + (threadIdx.x >> 7), d = threadIdx.x & 127;
  if (j >= v.M0) return;
  const int* koff = v.koff + (size_t)u * (v.Mcap + 1);
  const int* order = v.order + (size_t)u * v.Ncap;
  const int b = koff[j], e = koff[j + 1];
  if (e == b) return;
  double s = 0.0;
  for (int q = b; q < e; ++q) s += (double)load_elem(X, ((size_t)u * N0 + order[q]) * kHeadDim + d, v.dtype);
  unit_R(v, u)[r_index(j, d)] = (float)(s / (double)(e - b));
}

// One workgroup per unit: every empty cluster, in ascending id, takes the not-yet-taken point that is
// farthest from its own centre (ties to the lowest position).
__global__ __launch_bounds__(256) void kmeans_reseed_kernel(View v, const void* X, int N0) {
  __shared__ double sv[256];
  __shared__ int si[256];
  __shared__ int any_empty;
  const int u = blockIdx.x, tid = threadIdx.x;
  const int* koff = v.koff + (size_t)u * (v.Mcap + 1);
  double* dist = v.dist + (size_t)u * v.Ncap;
  if (tid == 0) any_empty = 0;
  __syncthreads();
  for (int j = tid; j < v.M0; j += 256)
    if (koff[j + 1] == koff[j]) any_empty = 1;
  __syncthreads();
  if (!any_empty) return;
  for (int j = 0; j < v.M0; ++j) {
    if (koff[j + 1] != koff[j]) continue;   // uniform across the block
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

// dist[i] = squared distance of point i to the (updated) centre of its own cluster
__global__ __launch_bounds__(256) void point_dist_kernel(View v, const void* X, int N0) {
  const int u = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
  if (i >= N0) return;
  const int j = v.labels[(size_t)u * v.Ncap + i];
  const float* R = unit_R(v, u);
  const size_t base = ((size_t)u * N0 + i) * kHeadDim;
  double acc = 0.0;
  for (int d = 0; d < kHeadDim; ++d) {
    const double t = (double)load_elem(X, base + d, v.dtype) - (double)R[r_index(j, d)];
    acc = fma(t, t, acc);
  }
  v.dist[(size_t)u * v.Ncap + i] = acc;
}

// One workgroup per unit: per-cluster n, M2 (members in order), page chains, tau, counters.
__global__ __launch_bounds__(1024) void finalize_kernel(View v, int N0) {
  __shared__ int sm[64];
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
      const int b = koff[j], e = koff[j + 1];
      double m2 = 0.0;
      for (int q = b; q < e; ++q) m2 += dist[order[q]];
      v.cn[cb + j] = e - b;
      v.cM2[cb + j] = m2;
      v.pg_off[cb + j] = base;
      for (int p = 0; p < kInlinePages; ++p) v.cpg[(cb + j) * kInlinePages + p] = p < np[k] ? base + p : -1;
      v.ctail[cb + j] = np[k] ? base + np[k] - 1 : -1;
      for (int p = 0; p < np[k]; ++p) v.pnext[(size_t)u * v.Pcap + base + p] = p + 1 < np[k] ? base + p + 1 : -1;
      base += np[k];
    } else {
      v.cn[cb + j] = 0; v.cM2[cb + j] = 0.0; v.ctail[cb + j] = -1;
      for (int p = 0; p < kInlinePages; ++p) v.cpg[(cb + j) * kInlinePages + p] = -1;
    }
    v.cb[cb + j] = 0; v.cflag[cb + j] = 0; v.in_req[cb + j] = 0;
  }
  __syncthreads();
  if (tid == 0) {
    double J = 0.0;
    for (int j = 0; j < v.M0; ++j) J += v.cM2[cb + j];
    v.tau[u] = (double)v.var_alpha * (J / (double)N0);
    v.M[u] = v.M0; v.N[u] = N0; v.err[u] = 0; v.nflag[u] = 0; v.n_sel[u] = 0; v.t_sel[u] = 0; v.n_list[u] = 0;
    v.ticket[u] = 0; v.bump[u] = total; v.free_top[u] = 0; v.last_assign[u] = -1;
    for (int k = 0; k < kCounters; ++k) v.counters[(size_t)u * kCounters + k] = 0;
  }
}

// 16 consecutive entries of the sorted order per workgroup: copy K and V into their page slots.
__global__ __launch_bounds__(256) void layout_copy_kernel(View v, const void* K, const void* V, int N0) {
  const int u = blockIdx.y, q = blockIdx.x * 16 + (threadIdx.x >> 4), c = threadIdx.x & 15;
  if (q >= N0) return;
  const int pos = v.order[(size_t)u * v.Ncap + q];
  const int j = v.labels[(size_t)u * v.Ncap + pos];
  const int rank = q - v.koff[(size_t)u * (v.Mcap + 1) + j];
  const int page = v.pg_off[(size_t)u * v.Mcap + j] + rank / kPageTokens, slot = rank % kPageTokens;
  char* pg = page_ptr(v, u, page);
  const size_t src = ((size_t)u * N0 + pos) * kHeadDim;
  for (int e = 0; e < 8; ++e) {
    const int d = c * 8 + e;
    copy_elem(pg, k_index(v.dtype, slot, d), K, src + d, v.dtype);
    copy_elem(pg, v_index(v.dtype, slot, d), V, src + d, v.dtype);
  }
  if (c == 0) v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + slot] = pos;
}

}  // namespace

hipError_t launch_build_index(const View& v, const void* K, const void* V, int N0, const int* init_idx, int iters,
                              void* ws, size_t ws_bytes, hipStream_t st) {
  // the whole workspace starts from zero: unused page slots must hold finite values
  fill32_kernel<<<2048, 256, 0, st>>>((uint32_t*)ws, ws_bytes / 4, 0u);
  kmeans_init_kernel<<<dim3(v.M0, v.U), 128, 0, st>>>(v, K, N0, init_idx);
  int Npad = 2, pos_bits = 1;
  while (Npad < N0) { Npad <<= 1; ++pos_bits; }
  const dim3 gpts((N0 + 255) / 256, v.U);
  for (int it = 0; it < iters; ++it) {
    kmeans_assign_f64_kernel<<<gpts, 256, 0, st>>>(v, K, N0);
    kmeans_sort_kernel<<<v.U, 1024, 0, st>>>(v, N0, Npad, pos_bits);
    kmeans_update_kernel<<<dim3((v.M0 + 1) / 2, v.U), 256, 0, st>>>(v, K, N0);
    if (it + 1 < iters) kmeans_reseed_kernel<<<v.U, 256, 0, st>>>(v, K, N0);
  }
  point_dist_kernel<<<gpts, 256, 0, st>>>(v, K, N0);
  finalize_kernel<<<v.U, 1024, 0, st>>>(v, N0);
  layout_copy_kernel<<<dim3((N0 + 15) / 16, v.U), 256, 0, st>>>(v, K, V, N0);
  return hipGetLastError();
}

}  // namespace dynakv
