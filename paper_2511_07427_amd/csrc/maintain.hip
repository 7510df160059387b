// Decode, second half of a step (Algorithm 1, decode block; Section 4.2):
//   append_kernel - nearest cluster (its own scan of the table, or the per-block results the score kernel of a
//                   whole-step call left), UpdateVar, threshold test, AddEntry + UpdateStats or buffer + flag;
//                   in a whole-step call the due splits follow in the same launch
//   split_kernel  - delayed splits of flagged clusters in the active set, then the forced split
//   export_kernel - snapshot of the index for tests
// One workgroup per unit; each unit's record is touched by that workgroup only.  All decisions are
// taken on float64 values summed in the fixed order of common.hpp, ties to the lowest index.
#include "split.hpp"
#include "score.hpp"

namespace dynakv {

namespace {

// ------------------------------------------------------------------------------------------- append
// How the kernel finds the nearest cluster:
//   kScanMean  its own float64 scan of the float32 means
//   kPreMean   the score kernel of the same step has left the nearest cluster of every block of 256 clusters
//              (float64, float32 means)
//   kPreZ      a matrix-core pass (the score kernel of the same step, or a pass of its own launched before this
//              kernel) has left z_j = <k, r~_j> - |r~_j|^2 / 2 of every cluster of the 16-bit search copy: the
//              largest is taken if the runner-up lies beyond the float32 error bound, otherwise the clusters within
//              the bound are compared in float64
// SPLIT: the unit's due splits follow in the same launch (the rest of a decode step on the separate-kernel path).
enum { kScanMean = 0, kPreMean = 1, kPreZ = 2 };
template <bool ON>
struct SplitLds {
  alignas(16) unsigned char raw[kSplitRaw];
  SplitWork wk;
};
template <>
struct SplitLds<false> {};
template <int DT, int MODE, bool SPLIT>
__global__ __launch_bounds__(256) void append_kernel(View v, const void* kin, const void* vin) {
  static_assert(kSplitThreads == 256, "split_unit is run by this kernel's whole workgroup");
  __shared__ AppendSmem a;
  __shared__ double sv[16];
  __shared__ int si[16];
  __shared__ float s2[16];
  __shared__ SplitLds<SPLIT> sp;
  const int u = blockIdx.x, tid = threadIdx.x;
  const float* R = unit_R(v, u);
  f4 row[8];
  if constexpr (MODE == kScanMean)
    if ((size_t)(tid | 63) * kHeadDim < v.Rstride) load_centroid_head(R, tid, row);     // requested before anything else
  const int M = v.M[u], N = v.N[u];
  if (N >= v.Ncap || M <= 0) {                          // refused (workgroup-uniform); due splits still run
    if (tid == 0) v.err[u] |= DYNAKV_ERR_TOKENS;
    if constexpr (SPLIT) {
      __syncthreads();
      split_unit<DT>(v, u, sp.raw, sp.wk, false);
    }
    return;
  }
  float k2 = 0.f;
  if (tid < kHeadDim) {
    const float kf = load_elem(kin, (size_t)u * kHeadDim + tid, v.dtype);
    a.kd[tid] = (double)kf;
    k2 = kf * kf;
  }
  __syncthreads();
  int j;
  if constexpr (MODE == kPreZ) {
    for (int o = 32; o > 0; o >>= 1) k2 += __shfl_xor(k2, o);
    if ((tid & 63) == 0) s2[tid >> 6] = k2;
    __syncthreads();
    const float kn = __builtin_sqrtf(s2[0] + s2[1]) * 1.0001f;
    const float* zd = v.zdist + (size_t)u * v.Mcap;
    // the matrix-core pass has left best / runner-up per 64 clusters
    float zb = -__builtin_inff(), z2 = -__builtin_inff();
    int jb = -1;
    const size_t wbase = (size_t)u * v.NB * 4;
    for (int w = tid; w * 64 < M; w += 256) merge_best2(zb, jb, z2, v.near_zb[wbase + w], v.near_zj[wbase + w], v.near_z2[wbase + w]);
    j = nearest_resolve<256>(v, u, M, zb, jb, z2, kn, __int_as_float(v.rmax2[u]), zd, unit_Rq(v, u), a.kd, sv, si, s2);
  } else {
    double best = __builtin_inf();
    int arg = -1;
    if constexpr (MODE == kPreMean) {
      for (int b = tid; b * 256 < M; b += 256) {          // blocks past the last cluster hold nothing of this step
        const double d = v.near_d[(size_t)u * v.NB + b];
        const int jj = v.near_j[(size_t)u * v.NB + b];
        if (arg < 0 || d < best || (d == best && jj < arg)) { best = d; arg = jj; }
      }
    } else {
      // nearest centre (squared Euclidean distance); lane = cluster, 16 contiguous bytes per lane and load
      for (int jj = tid; jj < M; jj += 256) {
        double dist[1];
        if (jj != tid) load_centroid_head(R, jj, row);
        centroid_sums<1>(R, jj, row, dist, [&](int d, float rv, double (&acc)[1]) __attribute__((always_inline)) {
          const double t = a.kd[d] - (double)rv;
          acc[0] = fma(t, t, acc[0]);
        });
        if (dist[0] < best || arg < 0) { best = dist[0]; arg = jj; }
      }
    }
    j = block_argmin<256>(best, arg, sv, si);
  }
  const AppendFetch f = append_fetch(v, u, j);
  append_commit<256>(v, u, j, M, N, kin, vin, a, f);
  if constexpr (SPLIT) {
    __syncthreads();                                    // the append's record is in place for the whole workgroup
    split_unit<DT>(v, u, sp.raw, sp.wk, false);
  }
}

// ------------------------------------------------------------------------------------------- chunked prefill
// Adaptive clustering through a long prefill (Section 7, Discussion 1): one workgroup per unit walks the chunk's n
// entries in order; each entry is assigned to its nearest cluster (matrix cores + float64 where needed for the
// 16-bit search copy, float64 scan for float32 means), appended with UpdateVar and the threshold test, and a
// flagged cluster is split at once (the view's B_max is 0).  K, V: [U][n][128].
template <int DT, bool MEAN>
__global__ __launch_bounds__(256) void extend_kernel(View v, const void* K, const void* V, int n) {
  __shared__ AppendSmem a;
  __shared__ double sv[16];
  __shared__ int si[16];
  __shared__ float s2[16];
  __shared__ int s_rmax2;
  __shared__ SplitLds<true> sp;
  constexpr bool BF = DT == DYNAKV_BF16;
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int es = elem_size(v.dtype);
  for (int t = 0; t < n; ++t) {
    // the entry's rows, as pointers that the per-unit indexing of the append (u * 128 + d) lands on
    const size_t shift = ((size_t)u * n + t - u) * kHeadDim * es;
    const void* kin = (const char*)K + shift;
    const void* vin = (const char*)V + shift;
    const int M = v.M[u], N = v.N[u];
    if (N >= v.Ncap || M <= 0) {                       // workgroup-uniform
      if (tid == 0) v.err[u] |= DYNAKV_ERR_TOKENS;
      return;
    }
    float k2 = 0.f;
    if (tid < kHeadDim) {
      const float kf = load_elem(kin, (size_t)u * kHeadDim + tid, v.dtype);
      a.kd[tid] = (double)kf;
      k2 = kf * kf;
    }
    if (tid == 0) s_rmax2 = 0;
    __syncthreads();
    int j;
    if constexpr (MEAN) {
      const float* R = unit_R(v, u);
      double best = __builtin_inf();
      int arg = -1;
      for (int jj = tid; jj < M; jj += 256) {
        f4 row[8];
        double dist[1];
        load_centroid_head(R, jj, row);
        centroid_sums<1>(R, jj, row, dist, [&](int d, float rv, double (&acc)[1]) __attribute__((always_inline)) {
          const double x = a.kd[d] - (double)rv;
          acc[0] = fma(x, x, acc[0]);
        });
        if (dist[0] < best || arg < 0) { best = dist[0]; arg = jj; }
      }
      j = block_argmin<256>(best, arg, sv, si);
    } else {
      for (int o = 32; o > 0; o >>= 1) k2 += __shfl_xor(k2, o);
      if (lane == 0) s2[wave] = k2;
      const uint4* tiles = (const uint4*)unit_Rq(v, u);
      float* zd = v.zdist + (size_t)u * v.Mcap;
      ScoreRows<1> A;
      load_score_rows<1>(A, 0, nullptr, (const char*)kin + (size_t)u * kHeadDim * es, 0, lane);    // row 0 = the entry
      float zb = -__builtin_inff(), z2 = -__builtin_inff(), rmax2 = 0.f;
      int jb = -1;
      const int ntile = (M + kTileClusters - 1) / kTileClusters;
      for (int T = wave; T < ntile; T += 4) {
        uint4 b[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) b[s] = tiles[((size_t)T * 4 + s) * 64 + lane];
        float red, kdot, nrm2;
        score_tile<BF, 1, true>(b, A, 0, DYNAKV_GROUP_MAX, lane, red, kdot, nrm2);
        const int jj = T * kTileClusters + lane;
        if (lane < kTileClusters && jj < M) {
          const float z = kdot - 0.5f * nrm2;
          zd[jj] = z;
          rmax2 = fmaxf(rmax2, nrm2);
          if (jb < 0 || z > zb) { z2 = jb < 0 ? z2 : zb; zb = z; jb = jj; }
          else z2 = fmaxf(z2, z);
        }
      }
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) rmax2 = fmaxf(rmax2, __shfl_xor(rmax2, o));
      if (lane == 0) atomicMax(&s_rmax2, __float_as_int(rmax2));
      __syncthreads();
      const float kn = __builtin_sqrtf(s2[0] + s2[1]) * 1.0001f;
      j = nearest_resolve<256>(v, u, M, zb, jb, z2, kn, __int_as_float(s_rmax2), zd, unit_Rq(v, u), a.kd, sv, si, s2);
    }
    const AppendFetch f = append_fetch(v, u, j);
    append_commit<256>(v, u, j, M, N, kin, vin, a, f);
    __syncthreads();                                    // the append's record is in place for the whole workgroup
    split_unit<DT>(v, u, sp.raw, sp.wk, false);
    __syncthreads();                                    // and the unit's counters for the next entry
  }
}

// Baseline without clustering (Section 8.1): the new entry becomes cluster M of its unit, its own representative.
__global__ __launch_bounds__(256) void append_token_kernel(View v, const void* kin, const void* vin) {
  __shared__ int s_page;
  const int u = blockIdx.x, tid = threadIdx.x;
  const int M = v.M[u], N = v.N[u];
  const size_t cbase = (size_t)u * v.Mcap;
  if (tid == 0) {
    int page = -1;
    if (N >= v.Ncap) v.err[u] |= DYNAKV_ERR_TOKENS;
    else if (M >= v.Mcap) v.err[u] |= DYNAKV_ERR_CLUSTERS;
    else {
      const int top = v.free_top[u], bump = v.bump[u];
      if (top > 0) { page = v.freelist[(size_t)u * v.Pcap + top - 1]; v.free_top[u] = top - 1; }
      else if (bump < v.Pcap) { page = bump; v.bump[u] = bump + 1; }
      else v.err[u] |= DYNAKV_ERR_TOKENS;
    }
    if (page >= 0) {
      v.pnext[(size_t)u * v.Pcap + page] = -1;
      for (int p = 0; p < kInlinePages; ++p) v.cpg[(cbase + M) * kInlinePages + p] = p == 0 ? page : -1;
      v.ctail[cbase + M] = page;
      v.cn[cbase + M] = 1; v.cb[cbase + M] = 0; v.csz[cbase + M] = 1; v.cflag[cbase + M] = 0; v.cM2[cbase + M] = 0.0;
      v.in_req[cbase + M] = 0;
      v.ppos[((size_t)u * v.Pcap + page) * kPageTokens] = N;
      v.last_assign[u] = M;
      v.M[u] = M + 1; v.N[u] = N + 1;
      if (v.local_W > 0) v.lcount[u] += 1;
    }
    s_page = page;
  }
  __syncthreads();
  const int page = s_page;
  if (page < 0) return;
  char* pg = page_ptr(v, u, page);
  if (tid < kHeadDim) {
    store_centroid(v, u, M, tid, load_elem(kin, (size_t)u * kHeadDim + tid, v.dtype));
    copy_elem(pg, k_index(v.dtype, 0, tid), kin, (size_t)u * kHeadDim + tid, v.dtype);
  } else {
    copy_elem(pg, v_index(v.dtype, 0, tid - kHeadDim), vin, (size_t)u * kHeadDim + tid - kHeadDim, v.dtype);
  }
}

// Local update (Section 2.3): the last W clusters of the unit, one entry each, are clustered among themselves by
// Lloyd's k-means into k clusters that take their place.  One workgroup per unit; keys staged in LDS as float32
// (exact for every storage type), float64 distances and sums, centres stored as float32.
__global__ __launch_bounds__(256) void local_recluster_kernel(View v, int iters) {
  __shared__ float x[kLocalWindowMax][kHeadDim + 1];
  __shared__ float r[kLocalClustersMax][kHeadDim];
  __shared__ double dist[kLocalWindowMax], m2[kLocalClustersMax];
  __shared__ int label[kLocalWindowMax], pos[kLocalWindowMax], opage[kLocalWindowMax], rank[kLocalWindowMax];
  __shared__ int cnt[kLocalClustersMax], pgbase[kLocalClustersMax + 1], npage[kLocalClustersMax + kLocalWindowMax / kPageTokens + 1];
  __shared__ int s_ok;
  const int u = blockIdx.x, tid = threadIdx.x, W = v.local_W, k = v.local_k;
  if (v.lcount[u] != W) return;                         // workgroup-uniform: an append of this window was refused
  const int M = v.M[u], base = M - W;
  const size_t cb = (size_t)u * v.Mcap;
  const int es = elem_size(v.dtype);
  if (tid < W) {
    const int pg = v.cpg[(cb + base + tid) * kInlinePages];
    opage[tid] = pg;
    pos[tid] = v.ppos[((size_t)u * v.Pcap + pg) * kPageTokens];
  }
  __syncthreads();
  for (int t = tid; t < W * kHeadDim; t += 256) x[t >> 7][t & 127] = page_key(v, u, opage[t >> 7], 0, t & 127);
  __syncthreads();
  for (int t = tid; t < k * kHeadDim; t += 256) r[t >> 7][t & 127] = x[(t >> 7) * W / k][t & 127];
  __syncthreads();
  for (int it = 0; it < iters; ++it) {
    if (tid < W) {                                      // nearest centre, ties to the lowest
      double best = __builtin_inf();
      int arg = 0;
      for (int j = 0; j < k; ++j) {
        double acc = 0.0;
#pragma unroll 8
        for (int d = 0; d < kHeadDim; ++d) {
          const double t = (double)x[tid][d] - (double)r[j][d];
          acc = fma(t, t, acc);
        }
        if (acc < best) { best = acc; arg = j; }
      }
      label[tid] = arg;
    }
    __syncthreads();
    for (int t = tid; t < k * kHeadDim; t += 256) {     // mean of the members; a centre without members stays
      const int j = t >> 7, d = t & 127;
      double sum = 0.0;
      int n = 0;
      for (int i = 0; i < W; ++i)
        if (label[i] == j) { sum += (double)x[i][d]; ++n; }
      if (n > 0) r[j][d] = (float)(sum / (double)n);
    }
    __syncthreads();
  }
  if (tid < W) {                                        // distance to the stored centre, place inside the cluster
    const int j = label[tid];
    double acc = 0.0;
    for (int d = 0; d < kHeadDim; ++d) {
      const double t = (double)x[tid][d] - (double)r[j][d];
      acc = fma(t, t, acc);
    }
    dist[tid] = acc;
    int rk = 0;
    for (int i = 0; i < tid; ++i) rk += label[i] == j;
    rank[tid] = rk;
  }
  __syncthreads();
  if (tid < k) {
    int n = 0;
    double s = 0.0;
    for (int i = 0; i < W; ++i)
      if (label[i] == tid) { ++n; s += dist[i]; }
    cnt[tid] = n; m2[tid] = s;
  }
  __syncthreads();
  if (tid == 0) {                                       // fresh pages for the k clusters; the W old pages are freed below
    int need = 0;
    for (int j = 0; j < k; ++j) { pgbase[j] = need; need += (cnt[j] + kPageTokens - 1) / kPageTokens; }
    pgbase[k] = need;
    int top = v.free_top[u], bump = v.bump[u];
    s_ok = top + (v.Pcap - bump) >= need;
    if (s_ok) {
      for (int p = 0; p < need; ++p) npage[p] = top > 0 ? v.freelist[(size_t)u * v.Pcap + --top] : bump++;
      v.free_top[u] = top; v.bump[u] = bump;
    } else {
      v.err[u] |= DYNAKV_ERR_TOKENS;
      v.lcount[u] = 0;
    }
  }
  __syncthreads();
  if (!s_ok) return;
  char* pool = v.pages + (size_t)u * v.Pcap * ((size_t)kPageElems * es);
  const int chunks = kHeadDim * es / 16;                // 16-byte chunks per row
  for (int t = tid; t < W * 2 * chunks; t += 256) {     // keys and values, row by row, old page -> new page
    const int i = t / (2 * chunks), c = t % (2 * chunks), kv = c / chunks, ch = c % chunks;
    const int j = label[i], dpage = npage[pgbase[j] + rank[i] / kPageTokens], slot = rank[i] % kPageTokens;
    const size_t so = (size_t)(kv ? v_index(v.dtype, 0, 0) : k_index(v.dtype, 0, 0)) * es + (size_t)ch * 16;
    const size_t dof = (size_t)(kv ? v_index(v.dtype, slot, 0) : k_index(v.dtype, slot, 0)) * es + (size_t)ch * 16;
    *(uint4*)(pool + (size_t)dpage * kPageElems * es + dof) = *(const uint4*)(pool + (size_t)opage[i] * kPageElems * es + so);
  }
  if (tid < W) {
    const int j = label[tid];
    v.ppos[((size_t)u * v.Pcap + npage[pgbase[j] + rank[tid] / kPageTokens]) * kPageTokens + rank[tid] % kPageTokens] = pos[tid];
  }
  for (int t = tid; t < k * kHeadDim; t += 256) store_centroid(v, u, base + (t >> 7), t & 127, r[t >> 7][t & 127]);
  if (tid < k) {
    const size_t cj = cb + base + tid;
    const int np = pgbase[tid + 1] - pgbase[tid];
    v.cn[cj] = cnt[tid]; v.cb[cj] = 0; v.csz[cj] = cnt[tid]; v.cflag[cj] = 0; v.cM2[cj] = m2[tid];
    for (int p = 0; p < kInlinePages; ++p) v.cpg[cj * kInlinePages + p] = p < np ? npage[pgbase[tid] + p] : -1;
    v.ctail[cj] = np ? npage[pgbase[tid] + np - 1] : -1;
    for (int p = 0; p < np; ++p) v.pnext[(size_t)u * v.Pcap + npage[pgbase[tid] + p]] = p + 1 < np ? npage[pgbase[tid] + p + 1] : -1;
  }
  for (int j = base + tid; j < M; j += 256) v.in_req[cb + j] = 0;
  __syncthreads();                                      // every copy has read its old page
  if (tid == 0) {
    int top = v.free_top[u];
    for (int i = 0; i < W; ++i) v.freelist[(size_t)u * v.Pcap + top++] = opage[i];
    v.free_top[u] = top;
    v.M[u] = base + k; v.lcount[u] = 0;
  }
}

// ------------------------------------------------------------------------------------------- split
template <int DT>
__global__ __launch_bounds__(kSplitThreads) void split_kernel(View v) {
  __shared__ __align__(16) unsigned char raw[kSplitRaw];
  __shared__ SplitWork wk;
  split_unit<DT>(v, blockIdx.x, raw, wk, false);
}

// ------------------------------------------------------------------------------------------- export
// One workgroup per unit.  Clusters are dealt in runs of `ch` consecutive ids per thread, so that the member
// lists come out cluster after cluster whatever the capacity.
__global__ __launch_bounds__(1024) void export_kernel(View v, dynakv_state_t o) {
  __shared__ int sm[64];
  const int u = blockIdx.x, tid = threadIdx.x;
  const int M = v.M[u], N = v.N[u];
  const size_t cbase = (size_t)u * v.Mcap;
  if (tid == 0) {
    if (o.n_clusters) o.n_clusters[u] = M;
    if (o.n_tokens) o.n_tokens[u] = N;
    if (o.error) o.error[u] = v.err[u];
    if (o.tau) o.tau[u] = v.tau[u];
    if (o.n_selected) o.n_selected[u] = v.n_sel[u];
    if (o.n_gathered) o.n_gathered[u] = v.t_sel[u];
    if (o.last_assign) o.last_assign[u] = v.last_assign[u];
    if (o.counters) {
      for (int k = 0; k < kCounters; ++k) o.counters[(size_t)u * kCounters + k] = v.counters[(size_t)u * kCounters + k];
      o.counters[(size_t)u * kCounters + 3] = v.bump[u] - v.free_top[u];
    }
  }
  for (int j = tid; j < v.Mcap; j += 1024) {
    const bool in = j < M;
    if (o.size) o.size[cbase + j] = in ? v.cn[cbase + j] : 0;
    if (o.buffered) o.buffered[cbase + j] = in ? v.cb[cbase + j] : 0;
    if (o.flag) o.flag[cbase + j] = in ? v.cflag[cbase + j] : 0;
    if (o.m2) o.m2[cbase + j] = in ? v.cM2[cbase + j] : 0.0;
    if (o.scores) o.scores[cbase + j] = in ? v.score[cbase + j] : 0.f;
    if (o.selected) o.selected[cbase + j] = j < v.n_sel[u] ? v.sel_ids[cbase + j] : -1;
    if (o.first_page) o.first_page[cbase + j] = in && v.cn[cbase + j] + v.cb[cbase + j] > 0 ? v.cpg[(cbase + j) * kInlinePages] : -1;
  }
  if (o.centroids) {
    const float* R = unit_R(v, u);
    for (size_t t = tid; t < (size_t)v.Mcap * kHeadDim; t += 1024) {
      const int j = (int)(t >> 7), d = (int)(t & 127);
      o.centroids[cbase * kHeadDim + t] = j < M ? R[r_index(j, d)] : 0.f;
    }
  }
  // member lists
  const int ch = (v.Mcap + 1023) / 1024;
  int tot = 0;
  for (int k = 0; k < ch; ++k) {
    const int j = tid * ch + k;
    if (j < M) tot += v.cn[cbase + j] + v.cb[cbase + j];
  }
  int total;
  int run = block_excl_scan(tot, sm, total);
  for (int k = 0; k < ch; ++k) {
    const int j = tid * ch + k;
    if (j >= v.Mcap) break;
    if (o.offsets) o.offsets[(size_t)u * (v.Mcap + 1) + j] = j < M ? run : total;
    if (j < M) { v.tok_off[cbase + j] = run; run += v.cn[cbase + j] + v.cb[cbase + j]; }
  }
  if (tid == 0 && o.offsets) o.offsets[(size_t)u * (v.Mcap + 1) + v.Mcap] = total;
  __syncthreads();
  const int es = elem_size(v.dtype);
  if (o.members || o.keys || o.values)
    for (int j = tid; j < M; j += 1024) {
      int w = v.tok_off[cbase + j], left = v.cn[cbase + j] + v.cb[cbase + j], page = -1;
      for (int k = 0; left > 0; ++k) {
        page = cluster_page(v, u, cbase + j, k, page);
        if (page < 0) break;
        const int nv = min(left, kPageTokens);
        const char* pg = page_ptr(v, u, page);
        for (int sl = 0; sl < nv; ++sl) {
          const int pos = v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + sl];
          if (o.members) o.members[(size_t)u * v.Ncap + w + sl] = pos;
          const size_t row = ((size_t)u * v.Ncap + pos) * kHeadDim * es;
          if (o.keys) {
            const uint4* src = (const uint4*)(pg + (size_t)k_index(v.dtype, sl, 0) * es);
            uint4* dst = (uint4*)((char*)o.keys + row);
            for (int c = 0; c < kHeadDim * es / 16; ++c) dst[c] = src[c];
          }
          if (o.values) {
            const uint4* src = (const uint4*)(pg + (size_t)v_index(v.dtype, sl, 0) * es);
            uint4* dst = (uint4*)((char*)o.values + row);
            for (int c = 0; c < kHeadDim * es / 16; ++c) dst[c] = src[c];
          }
        }
        w += nv; left -= nv;
      }
    }
  if (o.gathered) {
    const int nl = v.n_list[u];
    for (int w = tid; w < nl; w += 1024) {
      const int e = v.plist[(size_t)u * v.Lcap + w], t0 = v.plist_off[(size_t)u * v.Lcap + w];
      const int page = e >> 4, first = ((e >> 2) & 3) * 4, nv = (e & 3) + 1;
      for (int sl = 0; sl < nv; ++sl)
        o.gathered[(size_t)u * v.Ncap + t0 + sl] = v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + first + sl];
    }
  }
}

// ------------------------------------------------------------------------------------------- import
// First kernel of an import, one workgroup per unit: checks the snapshot's sizes, then writes every record of
// the unit (clusters, page chains, flagged list, active set, counters) and, for the copy kernel that follows,
// the cluster and the place of every token (labels / order / koff / pg_off, the scratch arrays of the prefill).
// v.nflagged[u] tells the copy kernel whether the unit was accepted.
__global__ __launch_bounds__(1024) void import_meta_kernel(View v, dynakv_state_t s) {
  __shared__ int sm[64];
  __shared__ int s_bad, s_nflag;
  const int u = blockIdx.x, tid = threadIdx.x;
  const size_t cbase = (size_t)u * v.Mcap;
  const int M = s.n_clusters[u], N = s.n_tokens[u];
  const int* off = s.offsets + (size_t)u * (v.Mcap + 1);
  const bool sane = M >= 1 && M <= v.Mcap && N >= 0 && N <= v.Ncap;
  if (tid == 0) { s_bad = 0; s_nflag = 0; }
  __syncthreads();
  const int ch = sane ? (M + 1023) / 1024 : 0;
  int tot = 0;
  if (sane) {
    if (tid == 0 && (off[0] != 0 || off[M] != N)) s_bad = 1;
    for (int k = 0; k < ch; ++k) {
      const int j = tid * ch + k;
      if (j >= M) break;
      const int n = s.size[cbase + j], b = s.buffered[cbase + j], m = off[j + 1] - off[j];
      if (n < 0 || b < 0 || m != n + b || (b != 0 && s.flag[cbase + j] == 0)) s_bad = 1;
      tot += (max(m, 0) + kPageTokens - 1) / kPageTokens;
    }
  }
  int total;
  int base = block_excl_scan(tot, sm, total);           // also the barrier behind s_bad
  if (!sane || s_bad || total > v.Pcap) {
    if (tid == 0) { atomicOr(&v.err[u], DYNAKV_ERR_IMPORT); v.nflagged[u] = 0; }
    return;
  }
  const int* mem = s.members + (size_t)u * v.Ncap;
  int* labels = v.labels + (size_t)u * v.Ncap;
  int* order = v.order + (size_t)u * v.Ncap;
  int* koff = v.koff + (size_t)u * (v.Mcap + 1);
  for (int k = 0; k < ch; ++k) {
    const int j = tid * ch + k;
    if (j >= M) break;
    const int m = off[j + 1] - off[j], np = (m + kPageTokens - 1) / kPageTokens;
    v.cn[cbase + j] = s.size[cbase + j]; v.cb[cbase + j] = s.buffered[cbase + j]; v.csz[cbase + j] = m;
    const int fl = s.flag[cbase + j] != 0;
    v.cflag[cbase + j] = fl; v.cM2[cbase + j] = s.m2[cbase + j];
    v.pg_off[cbase + j] = base; koff[j] = off[j];
    for (int p = 0; p < kInlinePages; ++p) v.cpg[(cbase + j) * kInlinePages + p] = p < np ? base + p : -1;
    v.ctail[cbase + j] = np ? base + np - 1 : -1;
    for (int p = 0; p < np; ++p) v.pnext[(size_t)u * v.Pcap + base + p] = p + 1 < np ? base + p + 1 : -1;
    if (fl) v.flist[cbase + atomicAdd(&s_nflag, 1)] = j;
    for (int q = off[j]; q < off[j + 1]; ++q) {
      const int pos = min(max(mem[q], 0), v.Ncap - 1);
      order[q] = pos; labels[pos] = j;
    }
    base += np;
  }
  for (int j = tid; j < v.Mcap; j += 1024) {
    v.in_req[cbase + j] = 0; v.score[cbase + j] = 0.f;
    if (j >= M) {
      v.cn[cbase + j] = 0; v.cb[cbase + j] = 0; v.csz[cbase + j] = 0; v.cflag[cbase + j] = 0; v.cM2[cbase + j] = 0.0;
      v.ctail[cbase + j] = -1;
      for (int p = 0; p < kInlinePages; ++p) v.cpg[(cbase + j) * kInlinePages + p] = -1;
    }
  }
  for (size_t t = tid; t < (size_t)M * kHeadDim; t += 1024)
    store_centroid(v, u, (int)(t >> 7), (int)(t & 127), s.centroids[cbase * kHeadDim + t]);
  __syncthreads();
  int nsel = 0;
  if (s.selected) {
    nsel = min(max(s.n_selected[u], 0), M);
    for (int i = tid; i < nsel; i += 1024) {
      const int id = min(max(s.selected[cbase + i], 0), M - 1);
      v.sel_ids[cbase + i] = id; v.in_req[cbase + id] = 1;
    }
  }
  if (tid == 0) {
    koff[M] = N;
    v.M[u] = M; v.N[u] = N; v.tau[u] = s.tau[u]; v.err[u] = 0; v.nflag[u] = s_nflag; v.n_sel[u] = nsel; v.t_sel[u] = 0;
    v.n_list[u] = 0; v.ticket[u] = 0; v.bump[u] = total; v.free_top[u] = 0; v.last_assign[u] = -1; v.lcount[u] = 0; v.rmax2[u] = 0;
    for (int k = 0; k < kCounters; ++k) v.counters[(size_t)u * kCounters + k] = 0;
    v.nflagged[u] = 1;
  }
}

// 16 consecutive places of the storage order per workgroup, 16 threads per entry: keys and values move from
// the snapshot (by position) into their cluster's pages as whole 16-byte chunks.
// `stride`: tokens per unit in K and V.
__global__ __launch_bounds__(256) void import_copy_kernel(View v, const void* K, const void* V, int stride) {
  const int u = blockIdx.y, q = blockIdx.x * 16 + (threadIdx.x >> 4), c = threadIdx.x & 15;
  if (!v.nflagged[u] || q >= v.N[u]) return;
  const int pos = v.order[(size_t)u * v.Ncap + q];
  const int j = v.labels[(size_t)u * v.Ncap + pos];
  const int rank = q - v.koff[(size_t)u * (v.Mcap + 1) + j];
  const int page = v.pg_off[(size_t)u * v.Mcap + j] + rank / kPageTokens, slot = rank % kPageTokens;
  char* pg = page_ptr(v, u, page);
  const size_t src = ((size_t)u * stride + pos) * kHeadDim + c * 8;
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

// ------------------------------------------------------------------------------------------- placement
// Correlation-aware placement (Section 5.1, Eq. 8).  F = P while counting: [U][M0][M0] float32 counts (exact).
__global__ __launch_bounds__(256) void cor_zero_kernel(float* F, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) F[i] = 0.f;
}
// After one reference retrieval: every ordered pair of different selected clusters is counted once.  One
// workgroup per unit; a pair belongs to one thread, and the launches of different queries follow each other.
__global__ __launch_bounds__(256) void cor_count_kernel(View v, float* F) {
  const int u = blockIdx.x, n = v.n_sel[u], M0 = v.M0;
  const int* ids = v.sel_ids + (size_t)u * v.Mcap;
  float* f = F + (size_t)u * M0 * M0;
  for (long long t = threadIdx.x; t < (long long)n * n; t += 256) {
    const int a = ids[t / n], b = ids[t % n];
    if (a != b && a < M0 && b < M0) f[(size_t)a * M0 + b] += 1.f;
  }
}
// One workgroup of 1024 threads per unit: the greedy chain on the counts, Eq. 8's normalisation, and the page
// table of the unit in chain order (pg_off / cpg / ctail / pnext), for the copy kernel that follows.
__global__ __launch_bounds__(1024) void cor_finish_kernel(View v, float* F, int* order_out, int n_tokens) {
  __shared__ float rowsum[kMaxInitClusters];
  __shared__ unsigned char placed[kMaxInitClusters];
  __shared__ float rv[16];
  __shared__ int ri[16];
  __shared__ double rt[16];
  __shared__ int s_last;
  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6, M0 = v.M0;
  const size_t cb = (size_t)u * v.Mcap;
  float* f = F + (size_t)u * M0 * M0;
  int* chain = v.tok_off + cb;
  const bool fresh = v.M[u] == M0 && v.N[u] == n_tokens && v.nflag[u] == 0 && v.free_top[u] == 0;
  if (!fresh) {                                            // workgroup-uniform
    if (tid == 0) { atomicOr(&v.err[u], DYNAKV_ERR_PLACE); v.nflagged[u] = 0; }
    return;
  }
  double tot = 0.0;
  for (int i = tid; i < M0; i += 1024) {
    float rs = 0.f;
    for (int j = 0; j < M0; ++j) rs += f[(size_t)i * M0 + j];          // whole numbers below 2^24: exact
    rowsum[i] = rs; placed[i] = 0;
    tot += (double)rs;
  }
  for (int o = 32; o > 0; o >>= 1) tot += __shfl_xor(tot, o);
  if (lane == 0) rt[w] = tot;
  __syncthreads();
  double total = 0.0;
  for (int k = 0; k < 16; ++k) total += rt[k];
  // arg-max over (value, id) pairs of the workgroup, lowest id among equals; id < 0: none
  auto argmax = [&](float val, int id) {
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(val, o);
      const int oi = __shfl_xor(id, o);
      if (oi >= 0 && (id < 0 || ov > val || (ov == val && oi < id))) { val = ov; id = oi; }
    }
    __syncthreads();
    if (lane == 0) { rv[w] = val; ri[w] = id; }
    __syncthreads();
    if (tid == 0) {
      float bv = rv[0]; int bi = ri[0];
      for (int k = 1; k < 16; ++k)
        if (ri[k] >= 0 && (bi < 0 || rv[k] > bv || (rv[k] == bv && ri[k] < bi))) { bv = rv[k]; bi = ri[k]; }
      s_last = bi;
    }
    __syncthreads();
    return s_last;
  };
  int last;
  {
    float bv = -1.f; int bi = -1;
    for (int i = tid; i < M0; i += 1024)
      if (rowsum[i] > bv) { bv = rowsum[i]; bi = i; }                  // ascending i per thread: the first maximum stays
    last = argmax(bv, bi);
  }
  for (int k = 0; k < M0; ++k) {
    if (tid == 0) { chain[k] = last; placed[last] = 1; }
    __syncthreads();
    if (k + 1 == M0) break;
    float bv = -1.f; int bi = -1;
    for (int j = tid; j < M0; j += 1024)
      if (!placed[j] && f[(size_t)last * M0 + j] > bv) { bv = f[(size_t)last * M0 + j]; bi = j; }
    last = argmax(bv, bi);
  }
  // Eq. 8
  const float inv = total > 0.0 ? (float)(1.0 / total) : 0.f;
  for (size_t t = tid; t < (size_t)M0 * M0; t += 1024) f[t] = total > 0.0 ? (float)((double)f[t] / total) : 0.f;
  (void)inv;
  if (order_out)
    for (int k = tid; k < M0; k += 1024) order_out[(size_t)u * M0 + k] = chain[k];
  // pages in chain order
  if (tid == 0) {
    int base = 0;
    for (int k = 0; k < M0; ++k) {
      const int j = chain[k];
      v.pg_off[cb + j] = base;
      base += (v.cn[cb + j] + kPageTokens - 1) / kPageTokens;
    }
    v.nflagged[u] = 1;
  }
  __syncthreads();
  for (int j = tid; j < M0; j += 1024) {
    const int np = (v.cn[cb + j] + kPageTokens - 1) / kPageTokens, base = v.pg_off[cb + j];
    for (int p = 0; p < kInlinePages; ++p) v.cpg[(cb + j) * kInlinePages + p] = p < np ? base + p : -1;
    v.ctail[cb + j] = np ? base + np - 1 : -1;
    for (int p = 0; p < np; ++p) v.pnext[(size_t)u * v.Pcap + base + p] = p + 1 < np ? base + p + 1 : -1;
  }
}
}  // namespace

// prescanned: the score kernel of the same step has already looked at the new key (launch_score_select with kin).
// Otherwise, with the 16-bit search copy, a matrix-core pass of its own comes first.
hipError_t launch_append(const View& v, const void* k, const void* val, bool prescanned, bool split, hipStream_t st) {
  if (v.token_level) {
    append_token_kernel<<<v.U, 256, 0, st>>>(v, k, val);
    return hipGetLastError();
  }
  if (!v.search_mean && !prescanned) {
    const hipError_t e = launch_near(v, k, st);
    if (e != hipSuccess) return e;
  }
  const int mode = !v.search_mean ? kPreZ : prescanned ? kPreMean : kScanMean;
#define DYNAKV_APPEND_M(DT, MODE)                                                         \
  do {                                                                                     \
    if (split) append_kernel<DT, MODE, true><<<v.U, 256, 0, st>>>(v, k, val);              \
    else append_kernel<DT, MODE, false><<<v.U, 256, 0, st>>>(v, k, val);                   \
  } while (0)
#define DYNAKV_APPEND(DT)                                                                  \
  do {                                                                                     \
    if (mode == kPreZ) DYNAKV_APPEND_M(DT, kPreZ);                                         \
    else if (mode == kPreMean) DYNAKV_APPEND_M(DT, kPreMean);                              \
    else DYNAKV_APPEND_M(DT, kScanMean);                                                   \
  } while (0)
  if (v.dtype == DYNAKV_F32) {
    if (prescanned) DYNAKV_APPEND_M(DYNAKV_F32, kPreMean);
    else DYNAKV_APPEND_M(DYNAKV_F32, kScanMean);
  }
  else if (v.dtype == DYNAKV_F16) DYNAKV_APPEND(DYNAKV_F16);
  else DYNAKV_APPEND(DYNAKV_BF16);
#undef DYNAKV_APPEND
#undef DYNAKV_APPEND_M
  return hipGetLastError();
}
hipError_t launch_local_recluster(const View& v, int iters, hipStream_t st) {
  local_recluster_kernel<<<v.U, 256, 0, st>>>(v, iters);
  return hipGetLastError();
}
hipError_t launch_extend(const View& v, const void* K, const void* V, int n, hipStream_t st) {
  if (v.dtype == DYNAKV_F32) extend_kernel<DYNAKV_F32, true><<<v.U, 256, 0, st>>>(v, K, V, n);
  else if (v.dtype == DYNAKV_F16) {
    if (v.search_mean) extend_kernel<DYNAKV_F16, true><<<v.U, 256, 0, st>>>(v, K, V, n);
    else extend_kernel<DYNAKV_F16, false><<<v.U, 256, 0, st>>>(v, K, V, n);
  } else {
    if (v.search_mean) extend_kernel<DYNAKV_BF16, true><<<v.U, 256, 0, st>>>(v, K, V, n);
    else extend_kernel<DYNAKV_BF16, false><<<v.U, 256, 0, st>>>(v, K, V, n);
  }
  return hipGetLastError();
}
hipError_t launch_split(const View& v, hipStream_t st) {
  if (v.dtype == DYNAKV_F32) split_kernel<DYNAKV_F32><<<v.U, kSplitThreads, 0, st>>>(v);
  else if (v.dtype == DYNAKV_F16) split_kernel<DYNAKV_F16><<<v.U, kSplitThreads, 0, st>>>(v);
  else split_kernel<DYNAKV_BF16><<<v.U, kSplitThreads, 0, st>>>(v);
  return hipGetLastError();
}
hipError_t launch_export(const View& v, const dynakv_state_t& dst, hipStream_t st) {
  export_kernel<<<v.U, 1024, 0, st>>>(v, dst);
  return hipGetLastError();
}
hipError_t launch_place(const View& v, const void* K, const void* V, int n_tokens, const void* Qref, int n_ref, int budget,
                        float* P, int* order, hipStream_t st) {
  const size_t n = (size_t)v.U * v.M0 * v.M0;
  cor_zero_kernel<<<1024, 256, 0, st>>>(P, n);
  const size_t qbytes = (size_t)v.U * v.G * kHeadDim * elem_size(v.dtype);
  for (int r = 0; r < n_ref; ++r) {
    const hipError_t e = launch_score_select(v, (const char*)Qref + (size_t)r * qbytes, budget, nullptr, st);
    if (e != hipSuccess) return e;
    cor_count_kernel<<<v.U, 256, 0, st>>>(v, P);
  }
  cor_finish_kernel<<<v.U, 1024, 0, st>>>(v, P, order, n_tokens);
  import_copy_kernel<<<dim3((n_tokens + 15) / 16, v.U), 256, 0, st>>>(v, K, V, n_tokens);
  return hipGetLastError();
}
hipError_t launch_import(const View& v, const dynakv_state_t& src, hipStream_t st) {
  import_meta_kernel<<<v.U, 1024, 0, st>>>(v, src);
  import_copy_kernel<<<dim3((v.Ncap + 15) / 16, v.U), 256, 0, st>>>(v, src.keys, src.values, v.Ncap);
  return hipGetLastError();
}

}  // namespace dynakv
