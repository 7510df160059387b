// Decode, second half of a step (Algorithm 1, decode block; Section 4.2):
//   append_kernel - nearest cluster, UpdateVar, threshold test, AddEntry + UpdateStats or buffer + flag
//   split_kernel  - delayed splits of flagged clusters in the active set, then the forced split
//   export_kernel - snapshot of the index for tests
// One workgroup per unit; each unit's record is touched by that workgroup only.  All decisions are
// taken on float64 values accumulated left to right, ties to the lowest index.
#include "append.hpp"

namespace dynakv {

namespace {

// ------------------------------------------------------------------------------------------- append
__global__ __launch_bounds__(256) void append_kernel(View v, const void* kin, const void* vin) {
  __shared__ AppendSmem a;
  __shared__ double sv[16];
  __shared__ int si[16];
  const int u = blockIdx.x, tid = threadIdx.x;
  float* R = unit_R(v, u);
  f4 row[8];
  if ((size_t)(tid | 63) * kHeadDim < v.Rstride) load_centroid_head(R, tid, row);   // requested before anything else
  const int M = v.M[u], N = v.N[u];
  if (N >= v.Ncap || M <= 0) {
    if (tid == 0) v.err[u] |= DYNAKV_ERR_TOKENS;
    return;
  }
  if (tid < kHeadDim) a.kd[tid] = (double)load_elem(kin, (size_t)u * kHeadDim + tid, v.dtype);
  __syncthreads();
  // nearest centre (squared Euclidean distance); lane = cluster, 16 contiguous bytes per lane and load
  double best = __builtin_inf();
  int arg = -1;
  for (int j = tid; j < M; j += 256) {
    if (j != tid) load_centroid_head(R, j, row);
    double dist[1];
    centroid_sums<1>(R, j, row, dist, [&](int d, float rv, double (&acc)[1]) __attribute__((always_inline)) {
      const double t = a.kd[d] - (double)rv;
      acc[0] = fma(t, t, acc[0]);
    });
    if (dist[0] < best || arg < 0) { best = dist[0]; arg = j; }
  }
  const int j = block_argmin<256>(best, arg, sv, si);
  append_commit<256>(v, u, j, M, N, kin, vin, a);
}

// ------------------------------------------------------------------------------------------- split
// Keys of the cluster being split are staged once in LDS (up to 128 members of a 16-bit type, 64 of
// float32; rows padded so that "lane = member" and "lane = coordinate" reads are both conflict-free);
// larger clusters fall back to reading their pages.
constexpr int kStageRow16 = kHeadDim + 8, kStageRow32 = kHeadDim + 4;
constexpr int kStageBytes = 128 * kStageRow16 * 2;

struct SplitSmem {
  int chain[kMaxSplitMembers / kPageTokens];      // pages of the cluster being split
  int newpg[kMaxSplitMembers / kPageTokens + 2];  // pages of the two children
  unsigned char side[kMaxSplitMembers];
  unsigned short perm[kMaxSplitMembers];           // members of the staying child in order, then of the moved one
  double cA[kHeadDim], cB[kHeadDim];
  float rA[kHeadDim], rB[kHeadDim];
  double sv[16];
  int si[16];
  double dl[128];                                  // member distances of a staged cluster
  int scan[64];
  int flag, count, nchain;
  int M, nflag, a_top, a_bump;                     // the unit's counters, held here for the whole kernel
  double m2[2];
  alignas(16) unsigned char stage[kStageBytes];
};

// Access to the keys of the members, by member index: 8 consecutive coordinates at a time, or one.
template <int DT, bool STAGED>
struct Keys {
  const View& v; const SplitSmem& s; int u;
  __device__ void get8(int i, int d8, float (&x)[8]) const {
    if constexpr (STAGED && DT == DYNAKV_F32) {
      const f4* p = (const f4*)((const float*)s.stage + i * kStageRow32 + d8 * 8);
      const f4 a = p[0], b = p[1];
#pragma unroll
      for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
    } else if constexpr (STAGED) {
      const uint4 w = *(const uint4*)((const uint16_t*)s.stage + i * kStageRow16 + d8 * 8);
      const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint16_t h = (uint16_t)(ww[e >> 1] >> ((e & 1) * 16));
        x[e] = DT == DYNAKV_F16 ? f16_to_float(h) : bf16_to_float(h);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = page_key(v, u, s.chain[i >> 4], i & 15, d8 * 8 + e);
    }
  }
  __device__ float get(int i, int d) const {
    if constexpr (STAGED && DT == DYNAKV_F32) return ((const float*)s.stage)[i * kStageRow32 + d];
    else if constexpr (STAGED) {
      const uint16_t h = ((const uint16_t*)s.stage)[i * kStageRow16 + d];
      return DT == DYNAKV_F16 ? f16_to_float(h) : bf16_to_float(h);
    } else return page_key(v, u, s.chain[i >> 4], i & 15, d);
  }
};

constexpr int kSplitThreads = 256;

// Arg-max over (value, index) pairs held one per thread of the whole block; ties go to the lowest index;
// index < 0 means "no candidate".  Wavefront shuffles first, then the 16 wavefront winners through LDS.
__device__ inline void block_argmax(double val, int idx, double* sv, int* si) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int o = 32; o > 0; o >>= 1) {
    const double ov = __shfl_xor(val, o);
    const int oi = __shfl_xor(idx, o);
    if (oi >= 0 && (idx < 0 || ov > val || (ov == val && oi < idx))) { val = ov; idx = oi; }
  }
  __syncthreads();
  if (lane == 0) { sv[w] = val; si[w] = idx; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < kSplitThreads / 64; ++k)
      if (si[k] >= 0 && (si[0] < 0 || sv[k] > sv[0] || (sv[k] == sv[0] && si[k] < si[0]))) { sv[0] = sv[k]; si[0] = si[k]; }
  }
  __syncthreads();
}

// Squared distances of member i to one or two centres (C = double or float) in the fixed summation order.
// Called by the four lanes of a quad at once: lane q accumulates blocks 4q..4q+3 (coordinates 32q..32q+31),
// the block sums are then added left to right across the quad; every lane returns the totals.
template <class K, class C>
__device__ inline void quad_sqdist(const K& ks, int i, int q, const C* cA, const C* cB, double& dA, double& dB) {
  double sa[4], sb[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    // every operand of the block is requested before the first use, so the LDS latency is paid once per block
    float x[8];
    C ca[8], cb[8];
    ks.get8(i, q * 4 + k, x);
#pragma unroll
    for (int e = 0; e < 8; ++e) { ca[e] = cA[(q * 4 + k) * 8 + e]; cb[e] = cB ? cB[(q * 4 + k) * 8 + e] : C(0); }
    asm volatile("" ::: "memory");
    double a = 0.0, b = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const double xd = (double)x[e];
      const double ta = xd - (double)ca[e];
      a = fma(ta, ta, a);
      if (cB) {
        const double tb = xd - (double)cb[e];
        b = fma(tb, tb, b);
      }
    }
    sa[k] = a; sb[k] = b;
  }
  dA = blocked16_quad(sa);
  dB = cB ? blocked16_quad(sb) : 0.0;
}

// Sum over r = 0..n-1, in that order, of key(r) for the r that use(r) accepts: eight operands are requested
// at a time (clamped, so the loads do not depend on the test), then added one by one; a rejected or
// out-of-range term adds +0.0, which leaves the float64 sum unchanged.
template <class Key, class Use>
__device__ inline double ordered_sum(int n, Key&& key, Use&& use) {
  double sum = 0.0;
  for (int r0 = 0; r0 < n; r0 += 8) {
    float x[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int r = min(r0 + k, n - 1);
      const float kv = key(r);
      x[k] = (r0 + k < n && use(r)) ? kv : 0.f;
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int k = 0; k < 8; ++k) sum += (double)x[k];
  }
  return sum;
}

// Arg-max of dist[0..n) (ties to the lowest index) by one thread, eight loads at a time; result in sv[0], si[0].
__device__ inline void serial_argmax(const double* dist, int n, double* sv, int* si) {
  __syncthreads();
  if (threadIdx.x == 0) {
    double bv = -1.0; int bi = -1;
    for (int r0 = 0; r0 < n; r0 += 8) {
      double x[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) x[k] = dist[min(r0 + k, n - 1)];
      asm volatile("" ::: "memory");
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (r0 + k < n && x[k] > bv) { bv = x[k]; bi = r0 + k; }
    }
    sv[0] = bv; si[0] = bi;
  }
  __syncthreads();
}

// Exact statistics of both children at once: members perm[0 .. nS) form cluster idS, perm[nS .. m) cluster idM
// (idM < 0: there is no second child).  Threads 0..127 own the coordinates of the first, 128..255 of the
// second.  float32 means go to rA / rB (LDS) and to the centroid table, M2 about those means to s.m2[].
template <class K>
__device__ inline void children_stats(const View& v, int u, SplitSmem& s, const K& ks, bool staged, int nS, int m,
                                      int idS, int idM) {
  const int tid = threadIdx.x, d = tid & (kHeadDim - 1), c = (tid >> 7) & 1;
  const int q0 = c ? nS : 0, q1 = c ? m : nS, id = c ? idM : idS;
  if (tid < 2 * kHeadDim) {
    float* r = c ? s.rB : s.rA;
    const double sum = ordered_sum(q1 - q0, [&](int r) { return ks.get(s.perm[q0 + r], d); }, [](int) { return true; });
    r[d] = q1 > q0 ? (float)(sum / (double)(q1 - q0)) : 0.f;
    if (id >= 0) unit_R(v, u)[r_index(id, d)] = r[d];
  }
  __syncthreads();
  double* dist = staged ? s.dl : v.dist + (size_t)u * v.Ncap;
  const int grp = tid >> 2, k = tid & 3;
  for (int base = 0; base < m; base += kSplitThreads / 4) {
    if (base + (int)((tid & ~63) >> 2) >= m) continue;      // this wavefront has no member
    const int q = base + grp, qc = min(q, m - 1);
    double da, db;
    quad_sqdist<K, float>(ks, s.perm[qc], k, qc < nS ? s.rA : s.rB, nullptr, da, db);
    if (k == 0 && q < m) dist[q] = da;
  }
  __syncthreads();
  if (d == 0 && tid < 2 * kHeadDim) {
    double acc = 0.0;
    for (int r0 = q0; r0 < q1; r0 += 8) {
      double x[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) x[k] = r0 + k < q1 ? dist[r0 + k] : 0.0;
      asm volatile("" ::: "memory");
#pragma unroll
      for (int k = 0; k < 8; ++k) acc += x[k];
    }
    s.m2[c] = acc;
  }
  __syncthreads();
}

// Splits cluster j of unit u (2-means; Algorithm 1 SplitCluster).  Whole block; all branches uniform.
template <int DT, bool STAGED>
__device__ __forceinline__ void split_cluster_impl(const View& v, int u, int j, int pos, int m, SplitSmem& s) {
  constexpr int NT = kSplitThreads;
  const int tid = threadIdx.x, grp = tid >> 2, kb = tid & 3;
  const int wave_first = (tid & ~63) >> 2;                    // first member this wavefront would take in a pass
  const size_t cbase = (size_t)u * v.Mcap;
  constexpr int kEs = DT == DYNAKV_F32 ? 4 : 2;
  constexpr int kChunks = kHeadDim * kEs / 16;                      // 16-byte chunks per key
  constexpr int kRowBytes = (DT == DYNAKV_F32 ? kStageRow32 : kStageRow16) * kEs;
  char* const pool = v.pages + (size_t)u * v.Pcap * ((size_t)kPageElems * kEs);
  const Keys<DT, STAGED> ks{v, s, u};
  // byte offset of 16-byte chunk c of the key in `slot` inside its page
  auto kchunk = [](int slot, int c) -> size_t {
    return (size_t)(DT == DYNAKV_F32 ? k_index32(slot, 4 * c) : k_index16(slot, 8 * c)) * kEs;
  };
  if constexpr (STAGED) {                  // one pass over the cluster's keys; every later pass reads LDS
    for (int t = tid; t < m * kChunks; t += NT) {
      const int i = t / kChunks, c = t % kChunks;
      *(uint4*)(s.stage + (size_t)i * kRowBytes + c * 16) =
          *(const uint4*)(pool + (size_t)s.chain[i >> 4] * (kPageElems * kEs) + kchunk(i & 15, c));
    }
    __syncthreads();
  }
  bool can_split = m >= 2;
  if (can_split) {
    // seeds: A = member farthest from the mean of all members, B = member farthest from A
    if (tid < kHeadDim) {
      const double sum = ordered_sum(m, [&](int i) { return ks.get(i, tid); }, [](int) { return true; });
      s.cA[tid] = sum / (double)m;
    }
    __syncthreads();
    double dummy;
    double* const seed_dist = STAGED ? s.dl : v.dist + (size_t)u * v.Ncap;
    for (int base = 0; base < m; base += NT / 4) {
      if (base + wave_first >= m) continue;
      const int i = base + grp;
      double t;
      quad_sqdist<decltype(ks), double>(ks, min(i, m - 1), kb, s.cA, nullptr, t, dummy);
      if (kb == 0 && i < m) seed_dist[i] = t;
    }
    serial_argmax(seed_dist, m, s.sv, s.si);
    const int a = s.si[0];
    __syncthreads();
    if (tid < kHeadDim) s.cB[tid] = (double)ks.get(a, tid);
    __syncthreads();
    for (int base = 0; base < m; base += NT / 4) {
      if (base + wave_first >= m) continue;
      const int i = base + grp;
      double t;
      quad_sqdist<decltype(ks), double>(ks, min(i, m - 1), kb, s.cB, nullptr, t, dummy);
      if (kb == 0 && i < m) seed_dist[i] = t;
    }
    serial_argmax(seed_dist, m, s.sv, s.si);
    const int b = s.si[0];
    const double db = s.sv[0];
    __syncthreads();
    can_split = db > 0.0;                 // false: all members identical
    if (can_split) {
      if (tid < kHeadDim) { s.cA[tid] = s.cB[tid]; }
      __syncthreads();
      if (tid < kHeadDim) s.cB[tid] = (double)ks.get(b, tid);
      for (int i = tid; i < m; i += NT) s.side[i] = 2;
      if (tid == 0) { s.flag = 0; s.count = 0; }
      __syncthreads();
      for (int it = 0; it < 16; ++it) {
        int changed = 0, na = 0;
        for (int base = 0; base < m; base += NT / 4) {
          if (base + wave_first >= m) continue;
          const int i = base + grp;
          double dA, dB;
          quad_sqdist<decltype(ks), double>(ks, min(i, m - 1), kb, s.cA, s.cB, dA, dB);
          if (kb == 0 && i < m) {
            const unsigned char ns = dA <= dB ? 0 : 1;   // tie -> side A
            changed |= ns != s.side[i];
            s.side[i] = ns;
            na += ns == 0;
          }
        }
        if (changed) s.flag = 1;
        if (na) atomicAdd(&s.count, na);
        __syncthreads();
        const int nA = s.count;
        const bool moved = s.flag != 0;
        __syncthreads();
        if (!moved) break;
        if (nA == 0 || nA == m) { can_split = false; break; }
        if (tid < 2 * kHeadDim) {
          const int d = tid & (kHeadDim - 1);
          const unsigned char mine = tid < kHeadDim ? 0 : 1;
          const double sum = ordered_sum(m, [&](int i) { return ks.get(i, d); }, [&](int i) { return s.side[i] == mine; });
          if (mine == 0) s.cA[d] = sum / (double)nA;
          else s.cB[d] = sum / (double)(m - nA);
        }
        if (tid == 0) { s.flag = 0; s.count = 0; }
        __syncthreads();
      }
    }
  }
  if (!can_split) {                       // unflag with exact statistics of the whole cluster
    for (int i = tid; i < m; i += NT) s.perm[i] = (unsigned short)i;
    __syncthreads();
    children_stats(v, u, s, ks, STAGED, m, m, j, -1);
    if (tid == 0) {
      v.cn[cbase + j] = m; v.cb[cbase + j] = 0; v.cflag[cbase + j] = 0; v.cM2[cbase + j] = s.m2[0];
      s.nflag -= 1;
      v.flist[cbase + pos] = v.flist[cbase + s.nflag];     // the last flagged id takes the freed place
      v.counters[(size_t)u * kCounters + 1] += 1;
    }
    __syncthreads();
    return;
  }
  const int M = s.M;
  if (M >= v.Mcap) {
    if (tid == 0) v.err[u] |= DYNAKV_ERR_CLUSTERS;
    return;
  }
  // stable partition: the child that holds the earliest entry keeps id j
  const unsigned char keep = s.side[0];
  const int chunk = (m + NT - 1) / NT;
  const int lo = min(m, tid * chunk), hi = min(m, lo + chunk);
  int mine = 0;
  for (int i = lo; i < hi; ++i) mine += s.side[i] == keep;
  int nS;
  int rs = block_excl_scan(mine, s.scan, nS);
  int rm = nS + lo - rs;
  for (int i = lo; i < hi; ++i) s.perm[s.side[i] == keep ? rs++ : rm++] = (unsigned short)i;
  const int nM = m - nS;
  const int pS = (nS + kPageTokens - 1) / kPageTokens, pM = (nM + kPageTokens - 1) / kPageTokens;
  const int need = pS + pM, top = s.a_top, bump = s.a_bump;
  if (top + (v.Pcap - bump) < need) {
    if (tid == 0) v.err[u] |= DYNAKV_ERR_TOKENS;
    return;
  }
  // fresh pages for both children (recycled pages first); the parent's pages are recycled afterwards
  const int from_free = min(need, top);
  for (int k = tid; k < need; k += NT)
    s.newpg[k] = k < from_free ? v.freelist[(size_t)u * v.Pcap + top - 1 - k] : bump + (k - from_free);
  __syncthreads();
  for (int k = tid; k < need; k += NT) {
    const bool last = k == pS - 1 || k == need - 1;
    v.pnext[(size_t)u * v.Pcap + s.newpg[k]] = last ? -1 : s.newpg[k + 1];
  }
  if (need > from_free) {                 // pages never used before are zeroed first
    constexpr int n16 = kPageElems * kEs / 16;
    for (int t = tid; t < (need - from_free) * n16; t += NT)
      ((uint4*)(pool + (size_t)s.newpg[from_free + t / n16] * (kPageElems * kEs)))[t % n16] = uint4{0, 0, 0, 0};
    __syncthreads();
  }
  // keys in 16-byte chunks, values element by element (their page layout interleaves four tokens)
  for (int t = tid; t < m * kChunks; t += NT) {
    const int q = t / kChunks, c = t % kChunks;
    const int i = s.perm[q];
    const int r = q < nS ? q : q - nS;
    const int dpage = s.newpg[(q < nS ? 0 : pS) + (r >> 4)];
    uint4 w;
    if constexpr (STAGED) w = *(const uint4*)(s.stage + (size_t)i * kRowBytes + c * 16);
    else w = *(const uint4*)(pool + (size_t)s.chain[i >> 4] * (kPageElems * kEs) + kchunk(i & 15, c));
    *(uint4*)(pool + (size_t)dpage * (kPageElems * kEs) + kchunk(r & 15, c)) = w;
  }
#pragma unroll 4
  for (int t = tid; t < m * kHeadDim; t += NT) {
    const int q = t >> 7, d = t & 127;
    const int i = s.perm[q];
    const int r = q < nS ? q : q - nS;
    const int dpage = s.newpg[(q < nS ? 0 : pS) + (r >> 4)];
    copy_elem(pool + (size_t)dpage * (kPageElems * kEs), v_index(DT, r & 15, d),
              pool + (size_t)s.chain[i >> 4] * (kPageElems * kEs), v_index(DT, i & 15, d), DT);
    if (d == 0)
      v.ppos[((size_t)u * v.Pcap + dpage) * kPageTokens + (r & 15)] =
          v.ppos[((size_t)u * v.Pcap + s.chain[i >> 4]) * kPageTokens + (i & 15)];
  }
  children_stats(v, u, s, ks, STAGED, nS, m, j, M);
  for (int k = tid; k < s.nchain; k += NT) v.freelist[(size_t)u * v.Pcap + (top - from_free) + k] = s.chain[k];
  if (tid < kInlinePages) {
    v.cpg[(cbase + j) * kInlinePages + tid] = tid < pS ? s.newpg[tid] : -1;
    v.cpg[(cbase + M) * kInlinePages + tid] = tid < pM ? s.newpg[pS + tid] : -1;
  }
  if (tid == 0) {
    v.cn[cbase + j] = nS; v.cb[cbase + j] = 0; v.cflag[cbase + j] = 0; v.cM2[cbase + j] = s.m2[0];
    v.ctail[cbase + j] = s.newpg[pS - 1];
    v.cn[cbase + M] = nM; v.cb[cbase + M] = 0; v.cflag[cbase + M] = 0; v.cM2[cbase + M] = s.m2[1];
    v.ctail[cbase + M] = s.newpg[pS + pM - 1];
    v.in_req[cbase + M] = 0;
    s.M = M + 1;
    s.a_top = top - from_free + s.nchain;
    s.a_bump = bump + (need - from_free);
    s.nflag -= 1;
    v.flist[cbase + pos] = v.flist[cbase + s.nflag];
    v.counters[(size_t)u * kCounters + 0] += 1;
  }
  __syncthreads();
}

template <int DT>
__device__ __forceinline__ void split_cluster(const View& v, int u, int j, int pos, SplitSmem& s) {
  const int tid = threadIdx.x;
  const size_t cbase = (size_t)u * v.Mcap;
  const int m = v.cn[cbase + j] + v.cb[cbase + j];
  if (m > kMaxSplitMembers) {
    if (tid == 0) v.err[u] |= DYNAKV_ERR_SPLIT_SIZE;
    return;
  }
  __syncthreads();
  const int npg = (m + kPageTokens - 1) / kPageTokens;
  if (tid < kInlinePages && tid < npg) s.chain[tid] = v.cpg[(cbase + j) * kInlinePages + tid];
  __syncthreads();
  if (tid == 0) {
    for (int k = kInlinePages; k < npg; ++k) s.chain[k] = v.pnext[(size_t)u * v.Pcap + s.chain[k - 1]];
    s.nchain = npg;
  }
  __syncthreads();
  if (m <= (DT == DYNAKV_F32 ? 64 : 128)) split_cluster_impl<DT, true>(v, u, j, pos, m, s);
  else split_cluster_impl<DT, false>(v, u, j, pos, m, s);
}

template <int DT>
__global__ __launch_bounds__(kSplitThreads) void split_kernel(View v) {
  constexpr int NT = kSplitThreads;
  __shared__ SplitSmem s;
  __shared__ int s_min;
  __shared__ long long s_tot;
  const int u = blockIdx.x, tid = threadIdx.x;
  if (v.nflag[u] == 0) return;
  const size_t cbase = (size_t)u * v.Mcap;
  const int M0 = v.M[u];
  if (tid == 0) { s.M = M0; s.nflag = v.nflag[u]; s.a_top = v.free_top[u]; s.a_bump = v.bump[u]; }
  // One loop, one call site: first the delayed splits (flagged clusters that the last retrieval selected, in
  // ascending id), then, once, the forced split of the fullest buffer if the buffers hold B_max entries.  Both
  // searches walk the list of flagged clusters, which holds a handful of ids.
  __syncthreads();
  int cursor = 0;
  bool forced_done = false;
  while (true) {
    int j = -1, pos = -1;
    const int nf = s.nflag;
    if (!forced_done) {
      if (tid == 0) s_min = 0x7FFFFFFF;
      __syncthreads();
      for (int i = tid; i < nf; i += NT) {
        const int c = v.flist[cbase + i];
        if (c >= cursor && c < M0 && (v.Bmax == 0 || v.in_req[cbase + c])) atomicMin(&s_min, c * kMaxClusters + i);
      }
      __syncthreads();
      if (s_min != 0x7FFFFFFF) { j = s_min / kMaxClusters; pos = s_min % kMaxClusters; }
      __syncthreads();
      if (j >= 0) cursor = j + 1;
    }
    if (j < 0) {
      if (forced_done) break;
      forced_done = true;
      if (!(v.Bmax > 0 && nf > 0)) break;
      if (tid == 0) s_tot = 0;
      __syncthreads();
      double bv = -1.0; int bi = -1;
      long long tot = 0;
      for (int i = tid; i < nf; i += NT) {
        const int c = v.flist[cbase + i];
        const int b = v.cb[cbase + c];
        tot += b;
        if ((double)b > bv || ((double)b == bv && c * kMaxClusters + i < bi)) { bv = (double)b; bi = c * kMaxClusters + i; }
      }
      if (tot) atomicAdd((unsigned long long*)&s_tot, (unsigned long long)tot);
      block_argmax(bv, bi, s.sv, s.si);
      const int arg = s.si[0];
      const long long total = s_tot;
      __syncthreads();
      if (!(arg >= 0 && total >= v.Bmax)) break;
      if (tid == 0) v.counters[(size_t)u * kCounters + 2] += 1;
      j = arg / kMaxClusters; pos = arg % kMaxClusters;
    }
    split_cluster<DT>(v, u, j, pos, s);
    __syncthreads();
    if (forced_done) break;
  }
  __syncthreads();
  if (tid == 0) { v.M[u] = s.M; v.nflag[u] = s.nflag; v.free_top[u] = s.a_top; v.bump[u] = s.a_bump; }
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

hipError_t launch_append(const View& v, const void* k, const void* val, hipStream_t st) {
  append_kernel<<<v.U, 256, 0, st>>>(v, k, val);
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
