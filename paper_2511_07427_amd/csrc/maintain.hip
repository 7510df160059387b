// Decode, second half of a step (Algorithm 1, decode block; Section 4.2):
//   append_kernel - nearest cluster (its own scan of the table, or the per-block results the score kernel of a
//                   whole-step call left), UpdateVar, threshold test, AddEntry + UpdateStats or buffer + flag;
//                   in a whole-step call the due splits follow in the same launch
//   split_kernel  - delayed splits of flagged clusters in the active set, then the forced split
//   export_kernel - snapshot of the index for tests
// One workgroup per unit; each unit's record is touched by that workgroup only.  All decisions are
// taken on float64 values summed in the fixed order of common.hpp, ties to the lowest index.
#include "split.hpp"

namespace dynakv {

namespace {

// ------------------------------------------------------------------------------------------- append
// PRE: the score kernel of the same step has left the nearest cluster of every block of 256 clusters.
// SPLIT: the unit's due splits follow in the same launch (the rest of a decode step on the separate-kernel path).
template <bool ON>
struct SplitLds {
  alignas(16) unsigned char raw[kSplitRaw];
  SplitWork wk;
};
template <>
struct SplitLds<false> {};
template <int DT, bool PRE, bool SPLIT>
__global__ __launch_bounds__(256) void append_kernel(View v, const void* kin, const void* vin) {
  static_assert(kSplitThreads == 256, "split_unit is run by this kernel's whole workgroup");
  __shared__ AppendSmem a;
  __shared__ double sv[16];
  __shared__ int si[16];
  __shared__ SplitLds<SPLIT> sp;
  const int u = blockIdx.x, tid = threadIdx.x;
  const float* R = unit_R(v, u);
  const uint16_t* Rq = unit_Rq(v, u);
  f4 row[8];
  uint4 hrow[1][4];
  double best = __builtin_inf();
  int arg = -1;
  if constexpr (PRE) {                                  // requested before anything else
    if (tid < kNearBlocks) { best = v.near_d[(size_t)u * kNearBlocks + tid]; arg = v.near_j[(size_t)u * kNearBlocks + tid]; }
  } else if ((size_t)(tid | 63) * kHeadDim < v.Rstride) {
    const int js[1] = {tid};
    if constexpr (DT == DYNAKV_F32) load_centroid_head(R, tid, row);
    else load_search_head<1>(Rq, js, hrow);
  }
  const int M = v.M[u], N = v.N[u];
  if (N >= v.Ncap || M <= 0) {                          // refused (workgroup-uniform); due splits still run
    if (tid == 0) v.err[u] |= DYNAKV_ERR_TOKENS;
    if constexpr (SPLIT) {
      __syncthreads();
      split_unit<DT>(v, u, sp.raw, sp.wk, false);
    }
    return;
  }
  if (tid < kHeadDim) a.kd[tid] = (double)load_elem(kin, (size_t)u * kHeadDim + tid, v.dtype);
  __syncthreads();
  if constexpr (PRE) {
    if (tid * 256 >= M) arg = -1;                       // blocks past the last cluster hold nothing of this step
  } else {
    // nearest centre (squared Euclidean distance); lane = cluster, 16 contiguous bytes per lane and load
    for (int j = tid; j < M; j += 256) {
      const int js[1] = {j};
      double dist[1][1];
      if constexpr (DT == DYNAKV_F32) {
        if (j != tid) load_centroid_head(R, j, row);
        centroid_sums<1>(R, j, row, dist[0], [&](int d, float rv, double (&acc)[1]) __attribute__((always_inline)) {
          const double t = a.kd[d] - (double)rv;
          acc[0] = fma(t, t, acc[0]);
        });
      } else {
        if (j != tid) load_search_head<1>(Rq, js, hrow);
        search_sums<1, 1, DT == DYNAKV_BF16>(Rq, js, hrow, dist,
            [&](int d, const float (&x)[1], double (&acc)[1][1]) __attribute__((always_inline)) {
          const double t = a.kd[d] - (double)x[0];
          acc[0][0] = fma(t, t, acc[0][0]);
        });
      }
      if (dist[0][0] < best || arg < 0) { best = dist[0][0]; arg = j; }
    }
  }
  const int j = block_argmin<256>(best, arg, sv, si);
  const AppendFetch f = append_fetch(v, u, j);
  append_commit<256>(v, u, j, M, N, kin, vin, a, f);
  if constexpr (SPLIT) {
    __syncthreads();                                    // the append's record is in place for the whole workgroup
    split_unit<DT>(v, u, sp.raw, sp.wk, false);
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
  }
  if (o.centroids) {
    const float* R = unit_R(v, u);
    for (size_t t = tid; t < (size_t)v.Mcap * kHeadDim; t += 1024) {
      const int j = (int)(t >> 7), d = (int)(t & 127);
      o.centroids[cbase * kHeadDim + t] = j < M ? R[r_index(j, d)] : 0.f;
    }
  }
  // member lists
  int sz[8], tot = 0;
  for (int k = 0; k < 8; ++k) {
    const int j = tid * 8 + k;
    sz[k] = j < M ? v.cn[cbase + j] + v.cb[cbase + j] : 0;
    tot += sz[k];
  }
  int total;
  int run = block_excl_scan(tot, sm, total);
  for (int k = 0; k < 8; ++k) {
    const int j = tid * 8 + k;
    if (j >= v.Mcap) break;
    if (o.offsets) o.offsets[(size_t)u * (v.Mcap + 1) + j] = j < M ? run : total;
    if (j < M) { v.tok_off[cbase + j] = run; run += sz[k]; }
  }
  if (tid == 0 && o.offsets) o.offsets[(size_t)u * (v.Mcap + 1) + v.Mcap] = total;
  __syncthreads();
  if (o.members)
    for (int j = tid; j < M; j += 1024) {
      int w = v.tok_off[cbase + j], left = v.cn[cbase + j] + v.cb[cbase + j], page = -1;
      for (int k = 0; left > 0; ++k) {
        page = cluster_page(v, u, cbase + j, k, page);
        if (page < 0) break;
        const int nv = min(left, kPageTokens);
        for (int sl = 0; sl < nv; ++sl)
          o.members[(size_t)u * v.Ncap + w + sl] = v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + sl];
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

}  // namespace

hipError_t launch_append(const View& v, const void* k, const void* val, bool prescanned, bool split, hipStream_t st) {
#define DYNAKV_APPEND(DT)                                                                    \
  do {                                                                                       \
    if (prescanned && split) append_kernel<DT, true, true><<<v.U, 256, 0, st>>>(v, k, val);  \
    else if (prescanned) append_kernel<DT, true, false><<<v.U, 256, 0, st>>>(v, k, val);     \
    else if (split) append_kernel<DT, false, true><<<v.U, 256, 0, st>>>(v, k, val);          \
    else append_kernel<DT, false, false><<<v.U, 256, 0, st>>>(v, k, val);                    \
  } while (0)
  if (v.dtype == DYNAKV_F32) DYNAKV_APPEND(DYNAKV_F32);
  else if (v.dtype == DYNAKV_F16) DYNAKV_APPEND(DYNAKV_F16);
  else DYNAKV_APPEND(DYNAKV_BF16);
#undef DYNAKV_APPEND
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

}  // namespace dynakv
