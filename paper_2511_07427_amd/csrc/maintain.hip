// Decode, second half of a step (Algorithm 1, decode block; Section 4.2):
//   append_kernel - nearest cluster, UpdateVar, threshold test, AddEntry + UpdateStats or buffer + flag
//   split_kernel  - delayed splits of flagged clusters in the active set, then the forced split
//   export_kernel - snapshot of the index for tests
// One workgroup per unit; each unit's record is touched by that workgroup only.  All decisions are
// taken on float64 values accumulated left to right, ties to the lowest index.
#include "common.hpp"

namespace dynakv {

namespace {

// Block-wide arg-min / arg-max over (value, index) pairs held one per thread; ties go to the lowest
// index; index < 0 means "no candidate".  256 threads.
template <bool MAX>
__device__ inline void block_arg_reduce(double val, int idx, double* sv, int* si) {
  const int tid = threadIdx.x;
  sv[tid] = val; si[tid] = idx;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) {
      const double ov = sv[tid + o];
      const int oi = si[tid + o];
      if (oi >= 0) {
        const bool better = si[tid] < 0 || (MAX ? ov > sv[tid] : ov < sv[tid]) || (ov == sv[tid] && oi < si[tid]);
        if (better) { sv[tid] = ov; si[tid] = oi; }
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------- append
__global__ __launch_bounds__(256) void append_kernel(View v, const void* kin, const void* vin) {
  __shared__ double kd[kHeadDim], r1[kHeadDim];
  __shared__ double sv[256];
  __shared__ int si[256];
  __shared__ int s_ok, s_commit, s_page, s_slot;
  const int u = blockIdx.x, tid = threadIdx.x;
  const int M = v.M[u], N = v.N[u];
  if (N >= v.Ncap || M <= 0) {
    if (tid == 0) v.err[u] |= DYNAKV_ERR_TOKENS;
    return;
  }
  if (tid < kHeadDim) kd[tid] = (double)load_elem(kin, (size_t)u * kHeadDim + tid, v.dtype);
  __syncthreads();
  const size_t cbase = (size_t)u * v.Mcap;
  // nearest centre (squared Euclidean distance)
  double best = __builtin_inf();
  int arg = -1;
  for (int j = tid; j < M; j += 256) {
    const f4* r = (const f4*)(v.R + (cbase + j) * kHeadDim);
    double acc = 0.0;
#pragma unroll 2
    for (int d4 = 0; d4 < kHeadDim / 4; ++d4) {
      const f4 rv = r[d4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const double t = kd[d4 * 4 + e] - (double)rv[e];
        acc = fma(t, t, acc);
      }
    }
    if (acc < best || arg < 0) { best = acc; arg = j; }
  }
  block_arg_reduce<false>(best, arg, sv, si);
  const int j = si[0];
  __syncthreads();
  if (tid == 0) {
    const int sz = v.cn[cbase + j] + v.cb[cbase + j];
    const int slot = sz % kPageTokens;
    int page = v.ctail[cbase + j];
    int ok = 1;
    if (slot == 0) {                      // no page yet, or the tail page is full
      const int np = alloc_page(v, u);
      if (np < 0) {
        v.err[u] |= DYNAKV_ERR_TOKENS;
        ok = 0;
      } else {
        v.pnext[(size_t)u * v.Pcap + np] = -1;
        if (sz == 0) v.chead[cbase + j] = np;
        else v.pnext[(size_t)u * v.Pcap + page] = np;
        v.ctail[cbase + j] = np;
        page = np;
      }
    }
    int commit = 0;
    if (ok) {
      v.last_assign[u] = j;
      if (v.cflag[cbase + j]) {
        v.cb[cbase + j] += 1;             // goes to the buffer of a flagged cluster
      } else {
        // UpdateVar: tentative n', r', M2' from (n, r, M2) and the new entry
        const float* r = v.R + (cbase + j) * kHeadDim;
        const int n1 = v.cn[cbase + j] + 1;
        double M2 = v.cM2[cbase + j];
        for (int d = 0; d < kHeadDim; ++d) {
          const double delta = kd[d] - (double)r[d];
          const double rd = (double)r[d] + delta / (double)n1;
          r1[d] = rd;
          M2 = fma(delta, kd[d] - rd, M2);
        }
        const double var1 = M2 / (double)n1;
        bool trig = false;
        if (n1 >= 2) {
          if (v.var_alpha > 0.f && var1 > v.tau[u]) trig = true;
          if (v.size_factor > 0.f && (double)n1 * (double)M > (double)v.size_factor * (double)(N + 1)) trig = true;
        }
        if (!trig) {
          v.cn[cbase + j] = n1;
          v.cM2[cbase + j] = M2;
          commit = 1;
        } else {
          v.cflag[cbase + j] = 1;
          v.cb[cbase + j] = 1;
          v.nflag[u] += 1;
        }
      }
      v.N[u] = N + 1;
      v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + slot] = N;
    }
    s_ok = ok; s_commit = commit; s_page = page; s_slot = slot;
  }
  __syncthreads();
  if (!s_ok) return;
  if (s_commit && tid < kHeadDim) v.R[(cbase + j) * kHeadDim + tid] = (float)r1[tid];
  char* pg = page_ptr(v, u, s_page);
  if (tid < kHeadDim) copy_elem(pg, k_index(v.dtype, s_slot, tid), kin, (size_t)u * kHeadDim + tid, v.dtype);
  else copy_elem(pg, v_index(v.dtype, s_slot, tid - kHeadDim), vin, (size_t)u * kHeadDim + tid - kHeadDim, v.dtype);
}

// ------------------------------------------------------------------------------------------- split
struct SplitSmem {
  int chain[kMaxSplitMembers / kPageTokens];      // pages of the cluster being split
  int newpg[kMaxSplitMembers / kPageTokens + 2];  // pages of the two children
  unsigned char side[kMaxSplitMembers];
  unsigned short rank[kMaxSplitMembers];           // rank of every member inside its child
  double cA[kHeadDim], cB[kHeadDim];
  float rA[kHeadDim], rB[kHeadDim];
  double sv[256];
  int si[256];
  int scan[64];
  int flag, count, nchain;
  double m2[2];
};

// squared distance of the key in (page, slot) to a float64 centre
__device__ inline double sqdist_page_d(const View& v, int u, int page, int slot, const double* c) {
  const char* pg = page_ptr(v, u, page);
  double acc = 0.0;
  for (int d = 0; d < kHeadDim; ++d) {
    const double t = (double)load_elem(pg, k_index(v.dtype, slot, d), v.dtype) - c[d];
    acc = fma(t, t, acc);
  }
  return acc;
}
__device__ inline double sqdist_page_f(const View& v, int u, int page, int slot, const float* c) {
  const char* pg = page_ptr(v, u, page);
  double acc = 0.0;
  for (int d = 0; d < kHeadDim; ++d) {
    const double t = (double)load_elem(pg, k_index(v.dtype, slot, d), v.dtype) - (double)c[d];
    acc = fma(t, t, acc);
  }
  return acc;
}

// Exact statistics of `n` members stored in order in pages pg[0..]: float32 mean into r (LDS) and to the
// cluster record `id`, M2 about that mean into *m2.  Threads [t0, t0+128) own the coordinates; the
// member distances go through dist[q0 .. q0+n).  Called by the whole block (contains barriers).
__device__ inline void child_stats(const View& v, int u, SplitSmem& s, const int* pg, int n, int id, float* r,
                                   int t0, int q0, double* m2) {
  const int tid = threadIdx.x;
  if (tid >= t0 && tid < t0 + kHeadDim) {
    const int d = tid - t0;
    double sum = 0.0;
    for (int i = 0; i < n; ++i) sum += (double)page_key(v, u, pg[i >> 4], i & 15, d);
    r[d] = n ? (float)(sum / (double)n) : 0.f;
    v.R[((size_t)u * v.Mcap + id) * kHeadDim + d] = r[d];
  }
  __syncthreads();
  double* dist = v.dist + (size_t)u * v.Ncap + q0;
  for (int i = tid; i < n; i += 256) dist[i] = sqdist_page_f(v, u, pg[i >> 4], i & 15, r);
  __syncthreads();
  if (tid == t0) {
    double acc = 0.0;
    for (int i = 0; i < n; ++i) acc += dist[i];
    *m2 = acc;
  }
  __syncthreads();
}

// Splits cluster j of unit u (2-means; Algorithm 1 SplitCluster).  Whole block; all branches uniform.
__device__ void split_cluster(const View& v, int u, int j, SplitSmem& s) {
  const int tid = threadIdx.x;
  const size_t cbase = (size_t)u * v.Mcap;
  const int m = v.cn[cbase + j] + v.cb[cbase + j];
  if (m > kMaxSplitMembers) {
    if (tid == 0) v.err[u] |= DYNAKV_ERR_SPLIT_SIZE;
    return;
  }
  __syncthreads();
  if (tid == 0) {
    int p = v.chead[cbase + j], k = 0;
    while (p >= 0 && k < kMaxSplitMembers / kPageTokens) { s.chain[k++] = p; p = v.pnext[(size_t)u * v.Pcap + p]; }
    s.nchain = k;
  }
  __syncthreads();
  bool can_split = m >= 2;
  if (can_split) {
    // seeds: A = member farthest from the mean of all members, B = member farthest from A
    if (tid < kHeadDim) {
      double sum = 0.0;
      for (int i = 0; i < m; ++i) sum += (double)page_key(v, u, s.chain[i >> 4], i & 15, tid);
      s.cA[tid] = sum / (double)m;
    }
    __syncthreads();
    double bv = -1.0; int bi = -1;
    for (int i = tid; i < m; i += 256) {
      const double t = sqdist_page_d(v, u, s.chain[i >> 4], i & 15, s.cA);
      if (t > bv) { bv = t; bi = i; }
    }
    block_arg_reduce<true>(bv, bi, s.sv, s.si);
    const int a = s.si[0];
    __syncthreads();
    if (tid < kHeadDim) s.cB[tid] = (double)page_key(v, u, s.chain[a >> 4], a & 15, tid);
    __syncthreads();
    bv = -1.0; bi = -1;
    for (int i = tid; i < m; i += 256) {
      const double t = sqdist_page_d(v, u, s.chain[i >> 4], i & 15, s.cB);
      if (t > bv) { bv = t; bi = i; }
    }
    block_arg_reduce<true>(bv, bi, s.sv, s.si);
    const int b = s.si[0];
    const double db = s.sv[0];
    __syncthreads();
    can_split = db > 0.0;                 // false: all members identical
    if (can_split) {
      if (tid < kHeadDim) { s.cA[tid] = s.cB[tid]; }
      __syncthreads();
      if (tid < kHeadDim) s.cB[tid] = (double)page_key(v, u, s.chain[b >> 4], b & 15, tid);
      for (int i = tid; i < m; i += 256) s.side[i] = 2;
      __syncthreads();
      for (int it = 0; it < 16; ++it) {
        if (tid == 0) { s.flag = 0; s.count = 0; }
        __syncthreads();
        int changed = 0, na = 0;
        for (int i = tid; i < m; i += 256) {
          const double dA = sqdist_page_d(v, u, s.chain[i >> 4], i & 15, s.cA);
          const double dB = sqdist_page_d(v, u, s.chain[i >> 4], i & 15, s.cB);
          const unsigned char ns = dA <= dB ? 0 : 1;   // tie -> side A
          changed |= ns != s.side[i];
          s.side[i] = ns;
          na += ns == 0;
        }
        if (changed) s.flag = 1;
        if (na) atomicAdd(&s.count, na);
        __syncthreads();
        const int nA = s.count;
        const bool moved = s.flag != 0;
        __syncthreads();
        if (!moved) break;
        if (nA == 0 || nA == m) { can_split = false; break; }
        {
          const int d = tid & (kHeadDim - 1);
          const unsigned char mine = tid < kHeadDim ? 0 : 1;
          double sum = 0.0;
          for (int i = 0; i < m; ++i)
            if (s.side[i] == mine) sum += (double)page_key(v, u, s.chain[i >> 4], i & 15, d);
          if (mine == 0) s.cA[d] = sum / (double)nA;
          else s.cB[d] = sum / (double)(m - nA);
        }
        __syncthreads();
      }
    }
  }
  if (!can_split) {                       // unflag with exact statistics of the whole cluster
    child_stats(v, u, s, s.chain, m, j, s.rA, 0, 0, &s.m2[0]);
    if (tid == 0) {
      v.cn[cbase + j] = m; v.cb[cbase + j] = 0; v.cflag[cbase + j] = 0; v.cM2[cbase + j] = s.m2[0];
      v.nflag[u] -= 1;
      v.counters[(size_t)u * kCounters + 1] += 1;
    }
    __syncthreads();
    return;
  }
  const int M = v.M[u];
  if (M >= v.Mcap) {
    if (tid == 0) v.err[u] |= DYNAKV_ERR_CLUSTERS;
    return;
  }
  // stable partition: the child that holds the earliest entry keeps id j
  const unsigned char keep = s.side[0];
  const int chunk = (m + 255) / 256;
  const int lo = min(m, tid * chunk), hi = min(m, lo + chunk);
  int mine = 0;
  for (int i = lo; i < hi; ++i) mine += s.side[i] == keep;
  int nS;
  int rs = block_excl_scan(mine, s.scan, nS);
  int rm = lo - rs;
  for (int i = lo; i < hi; ++i) s.rank[i] = (unsigned short)(s.side[i] == keep ? rs++ : rm++);
  const int nM = m - nS;
  const int pS = (nS + kPageTokens - 1) / kPageTokens, pM = (nM + kPageTokens - 1) / kPageTokens;
  if (pages_available(v, u) < pS + pM) {
    if (tid == 0) v.err[u] |= DYNAKV_ERR_TOKENS;
    return;
  }
  __syncthreads();
  if (tid == 0) {
    for (int k = 0; k < pS + pM; ++k) s.newpg[k] = alloc_page(v, u);
    for (int k = 0; k < pS; ++k) v.pnext[(size_t)u * v.Pcap + s.newpg[k]] = k + 1 < pS ? s.newpg[k + 1] : -1;
    for (int k = 0; k < pM; ++k) v.pnext[(size_t)u * v.Pcap + s.newpg[pS + k]] = k + 1 < pM ? s.newpg[pS + k + 1] : -1;
  }
  __syncthreads();
  // move every entry to its child's pages (both children get fresh pages; the old ones are recycled)
  for (int i = 0; i < m; ++i) {
    const int r = s.rank[i];
    const int dpage = s.newpg[(s.side[i] == keep ? 0 : pS) + (r >> 4)], dslot = r & 15;
    const int spage = s.chain[i >> 4], sslot = i & 15;
    char* dp = page_ptr(v, u, dpage);
    const char* sp = page_ptr(v, u, spage);
    if (tid < kHeadDim) copy_elem(dp, k_index(v.dtype, dslot, tid), sp, k_index(v.dtype, sslot, tid), v.dtype);
    else copy_elem(dp, v_index(v.dtype, dslot, tid - kHeadDim), sp, v_index(v.dtype, sslot, tid - kHeadDim), v.dtype);
    if (tid == 0)
      v.ppos[((size_t)u * v.Pcap + dpage) * kPageTokens + dslot] = v.ppos[((size_t)u * v.Pcap + spage) * kPageTokens + sslot];
  }
  __syncthreads();
  child_stats(v, u, s, s.newpg, nS, j, s.rA, 0, 0, &s.m2[0]);
  child_stats(v, u, s, s.newpg + pS, nM, M, s.rB, kHeadDim, nS, &s.m2[1]);
  if (tid == 0) {
    v.cn[cbase + j] = nS; v.cb[cbase + j] = 0; v.cflag[cbase + j] = 0; v.cM2[cbase + j] = s.m2[0];
    v.chead[cbase + j] = s.newpg[0]; v.ctail[cbase + j] = s.newpg[pS - 1];
    v.cn[cbase + M] = nM; v.cb[cbase + M] = 0; v.cflag[cbase + M] = 0; v.cM2[cbase + M] = s.m2[1];
    v.chead[cbase + M] = s.newpg[pS]; v.ctail[cbase + M] = s.newpg[pS + pM - 1];
    v.in_req[cbase + M] = 0;
    v.M[u] = M + 1;
    for (int k = 0; k < s.nchain; ++k) free_page(v, u, s.chain[k]);
    v.nflag[u] -= 1;
    v.counters[(size_t)u * kCounters + 0] += 1;
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void split_kernel(View v) {
  __shared__ SplitSmem s;
  __shared__ int s_min;
  __shared__ long long s_tot;
  const int u = blockIdx.x, tid = threadIdx.x;
  if (v.nflag[u] == 0) return;
  const size_t cbase = (size_t)u * v.Mcap;
  const int M0 = v.M[u];
  // delayed splits: flagged clusters that the last retrieval selected, ascending id
  int cursor = 0;
  while (true) {
    if (tid == 0) s_min = 0x7FFFFFFF;
    __syncthreads();
    for (int j = cursor + tid; j < M0; j += 256)
      if (v.cflag[cbase + j] && (v.Bmax == 0 || v.in_req[cbase + j])) { atomicMin(&s_min, j); break; }
    __syncthreads();
    const int j = s_min;
    __syncthreads();
    if (j == 0x7FFFFFFF) break;
    split_cluster(v, u, j, s);
    __syncthreads();
    cursor = j + 1;
  }
  // forced split once the buffers hold B_max entries: the flagged cluster with the fullest buffer
  if (v.Bmax > 0) {
    const int M = v.M[u];
    if (tid == 0) s_tot = 0;
    __syncthreads();
    double bv = -1.0; int bi = -1;
    long long tot = 0;
    for (int j = tid; j < M; j += 256)
      if (v.cflag[cbase + j]) {
        const int b = v.cb[cbase + j];
        tot += b;
        if ((double)b > bv) { bv = (double)b; bi = j; }
      }
    if (tot) atomicAdd((unsigned long long*)&s_tot, (unsigned long long)tot);
    block_arg_reduce<true>(bv, bi, s.sv, s.si);
    const int arg = s.si[0];
    const long long total = s_tot;
    __syncthreads();
    if (arg >= 0 && total >= v.Bmax) {
      if (tid == 0) v.counters[(size_t)u * kCounters + 2] += 1;
      split_cluster(v, u, arg, s);
    }
  }
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
  if (o.centroids)
    for (size_t t = tid; t < (size_t)v.Mcap * kHeadDim; t += 1024)
      o.centroids[cbase * kHeadDim + t] = t < (size_t)M * kHeadDim ? v.R[cbase * kHeadDim + t] : 0.f;
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
      int w = v.tok_off[cbase + j], left = v.cn[cbase + j] + v.cb[cbase + j], page = v.chead[cbase + j];
      while (left > 0 && page >= 0) {
        const int nv = min(left, kPageTokens);
        for (int sl = 0; sl < nv; ++sl)
          o.members[(size_t)u * v.Ncap + w + sl] = v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + sl];
        w += nv; left -= nv;
        page = v.pnext[(size_t)u * v.Pcap + page];
      }
    }
  if (o.gathered) {
    const int nl = v.n_list[u];
    for (int w = tid; w < nl; w += 1024) {
      const int e = v.plist[(size_t)u * v.Pcap + w], page = e >> 5, nv = e & 31, t0 = v.plist_off[(size_t)u * v.Pcap + w];
      for (int sl = 0; sl < nv; ++sl)
        o.gathered[(size_t)u * v.Ncap + t0 + sl] = v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + sl];
    }
  }
}

}  // namespace

hipError_t launch_append(const View& v, const void* k, const void* val, hipStream_t st) {
  append_kernel<<<v.U, 256, 0, st>>>(v, k, val);
  return hipGetLastError();
}
hipError_t launch_split(const View& v, hipStream_t st) {
  split_kernel<<<v.U, 256, 0, st>>>(v);
  return hipGetLastError();
}
hipError_t launch_export(const View& v, const dynakv_state_t& dst, hipStream_t st) {
  export_kernel<<<v.U, 1024, 0, st>>>(v, dst);
  return hipGetLastError();
}

}  // namespace dynakv
