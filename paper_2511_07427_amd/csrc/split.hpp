// Cluster splitting of a decode step (Algorithm 1, decode block; Section 4.2): shared by the stand-alone split
// kernel and by the kernel that runs a whole decode step per unit.
#pragma once
#include "append.hpp"

namespace dynakv {

namespace {

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
  alignas(16) float rA[kHeadDim], rB[kHeadDim];
  double tpart[4];                                 // per-wavefront parts of a sum over the coordinates, two rounds' worth
  double mu2[2];                                   // |mean of the members|^2, in two parts
  int nchg[2];                                     // members that changed side in a round (two rounds' worth)
  unsigned short chg[2][kMaxSplitMembers];         // who they are: member | what happens to the sums of side A << 12
  double sv[16];
  int si[16];
  double dl[128];                                  // member distances of a staged cluster
  int scan[64];
  int flag, count, nchain;
  int did_split;                                   // thread 0 only: the last split_cluster call split its cluster
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

// Side of member i in a round of the 2-means: A (0) if |x - cA|^2 <= |x - cB|^2, which is <x, w> <= t with
// w = cB - cA and t = (|cB|^2 - |cA|^2) / 2 (ties to A).  Called by the four lanes of a quad at once (lane q takes
// coordinates 32 q .. 32 q + 31); every lane gets the side.  The inner product is first taken in float32 against wf
// (= w rounded to float32); only if it lies within eps of t, the bound on what float32 can have changed, it is
// retaken in float64 against wd.
template <class K>
__device__ inline unsigned char quad_side(const K& ks, int i, int q, const float* wf, const double* wd, double t, float eps) {
  float x[4][8];
#pragma unroll
  for (int k = 0; k < 4; ++k) ks.get8(i, q * 4 + k, x[k]);
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const f4 a = *(const f4*)(wf + (q * 4 + k) * 8), b = *(const f4*)(wf + (q * 4 + k) * 8 + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { s = fmaf(x[k][e], a[e], s); s = fmaf(x[k][4 + e], b[e], s); }
  }
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  const float tf = (float)t;
  if (fabsf(s - tf) > eps) return s <= tf ? 0 : 1;            // uniform over the quad
  double sd = 0.0;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) sd = fma((double)x[k][e], wd[(q * 4 + k) * 8 + e], sd);
  sd += __shfl_xor(sd, 1);
  sd += __shfl_xor(sd, 2);
  return sd <= t ? 0 : 1;
}
// Bound for quad_side: float32 accumulation of 128 products (128 * 2^-24 |x| |w|, doubled for the rounding of w and
// of the products' partial sums across the quad) plus the rounding of t.  xmax >= every member's norm, wmax >= |w|.
__device__ inline float side_eps(float xmax, float wmax, double t) {
  return 1.53e-5f * xmax * wmax + 2.4e-7f * fabsf((float)t) + 1e-30f;
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
    if (id >= 0) store_centroid(v, u, id, d, r[d]);
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
    double total_d = 0.0;                 // thread d < 128: sum of coordinate d over all members
    if (tid < kHeadDim) {
      total_d = ordered_sum(m, [&](int i) { return ks.get(i, tid); }, [](int) { return true; });
      const double mu = total_d / (double)m;
      s.cA[tid] = mu;
      double mu2 = mu * mu;
      for (int o = 32; o > 0; o >>= 1) mu2 += __shfl_xor(mu2, o);
      if ((tid & 63) == 0) s.mu2[tid >> 6] = mu2;                    // |mean|^2, for the rounding bound of the rounds
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
    const float spread = (float)sqrt(s.sv[0]) * 1.0001f;                 // every member lies this close to the mean
    const float xmax = spread + (float)sqrt(s.mu2[0] + s.mu2[1]) * 1.0001f;
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
      // Lloyd rounds.  Thread d < 128 owns coordinate d: both centres and the sum of side A (registers); side B is
      // what is left of the total.  A round's side test is one inner product with w = cB - cA per member
      // (quad_side): w goes to s.cA (float64) and s.rA (float32).  Members that change side are listed, and the
      // sums follow the list instead of being formed anew (float64 sums of 16-bit values: exact, or very nearly).
      // Every member and every centre lies within sqrt(dmax) of the mean.  Two barriers per round.
      double ca = 0.0, cb = 0.0, sa = 0.0;
      if (tid < kHeadDim) { ca = s.cB[tid]; cb = (double)ks.get(b, tid); }
      for (int i = tid; i < m; i += NT) s.side[i] = 2;
      if (tid == 0) { s.nchg[0] = 0; s.nchg[1] = 0; }
      auto publish = [&](int slot) __attribute__((always_inline)) {       // w and t of the coming round
        if (tid < kHeadDim) {
          const double w = cb - ca;
          s.cA[tid] = w; s.rA[tid] = (float)w;
          double tp = 0.5 * (cb * cb - ca * ca);
          for (int o = 32; o > 0; o >>= 1) tp += __shfl_xor(tp, o);
          if ((tid & 63) == 0) s.tpart[slot * 2 + (tid >> 6)] = tp;
        }
      };
      publish(0);
      __syncthreads();
      int nA = 0;
      for (int it = 0; it < 16; ++it) {
        const int p = it & 1;
        const double t = s.tpart[p * 2] + s.tpart[p * 2 + 1];
        const float eps = side_eps(xmax, 2.f * spread, t);
        for (int base = 0; base < m; base += NT / 4) {
          if (base + wave_first >= m) continue;
          const int i = base + grp;
          const unsigned char ns = quad_side(ks, min(i, m - 1), kb, s.rA, s.cA, t, eps);
          if (kb == 0 && i < m) {
            const unsigned char old = s.side[i];
            if (ns != old) {     // 0: joins side A; 1: leaves nothing (first round, side B); 2: leaves side A
              s.side[i] = ns;
              const int code = ns == 0 ? 0 : old == 2 ? 1 : 2;
              s.chg[p][atomicAdd(&s.nchg[p], 1)] = (unsigned short)(i | (code << 12));
            }
          }
        }
        __syncthreads();
        const int nc = s.nchg[p];
        if (nc == 0) break;                                  // no member moved
        for (int e = 0; e < nc; ++e) {
          const int code = s.chg[p][e] >> 12;
          nA += code == 0 ? 1 : code == 2 ? -1 : 0;
        }
        if (nA == 0 || nA == m) { can_split = false; break; }
        if (tid < kHeadDim) {
          for (int e0 = 0; e0 < nc; e0 += 8) {               // eight members requested at a time
            float x[8];
            int cd[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const int en = s.chg[p][min(e0 + k, nc - 1)];
              cd[k] = e0 + k < nc ? en >> 12 : 1;
              x[k] = ks.get(en & 0xFFF, tid);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) sa += cd[k] == 0 ? (double)x[k] : cd[k] == 2 ? -(double)x[k] : 0.0;
          }
          ca = sa / (double)nA;
          cb = (total_d - sa) / (double)(m - nA);
        }
        if (tid == 0) s.nchg[p ^ 1] = 0;
        publish(p ^ 1);
        __syncthreads();
      }
    }
  }
  if (!can_split) {                       // unflag with exact statistics of the whole cluster
    for (int i = tid; i < m; i += NT) s.perm[i] = (unsigned short)i;
    __syncthreads();
    children_stats(v, u, s, ks, STAGED, m, m, j, -1);
    if (tid == 0) {
      v.cn[cbase + j] = m; v.csz[cbase + j] = m; v.cb[cbase + j] = 0; v.cflag[cbase + j] = 0; v.cM2[cbase + j] = s.m2[0];
      s.nflag -= 1;
      s.did_split = 0;
      v.flist[cbase + pos] = v.flist[cbase + s.nflag];     // the last flagged id takes the freed place
      count(v, u, 1, 1);
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
  int rs = block_excl_scan(mine, s.scan, nS, kSplitThreads / 64);
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
  // keys and values in 16-byte chunks of their rows (the V row of a slot lies one K region after its K row)
  constexpr size_t kVRegion = (size_t)kPageTokens * kHeadDim * kEs;
#pragma unroll 2
  for (int t = tid; t < m * kChunks; t += NT) {
    const int q = t / kChunks, c = t % kChunks;
    const int i = s.perm[q];
    const int r = q < nS ? q : q - nS;
    const int dpage = s.newpg[(q < nS ? 0 : pS) + (r >> 4)];
    const char* src = pool + (size_t)s.chain[i >> 4] * (kPageElems * kEs) + kchunk(i & 15, c);
    char* dst = pool + (size_t)dpage * (kPageElems * kEs) + kchunk(r & 15, c);
    uint4 w;
    if constexpr (STAGED) w = *(const uint4*)(s.stage + (size_t)i * kRowBytes + c * 16);
    else w = *(const uint4*)src;
    const uint4 x = *(const uint4*)(src + kVRegion);
    *(uint4*)dst = w;
    *(uint4*)(dst + kVRegion) = x;
    if (c == 0)
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
    v.cn[cbase + j] = nS; v.csz[cbase + j] = nS; v.cb[cbase + j] = 0; v.cflag[cbase + j] = 0; v.cM2[cbase + j] = s.m2[0];
    v.ctail[cbase + j] = s.newpg[pS - 1];
    v.cn[cbase + M] = nM; v.csz[cbase + M] = nM; v.cb[cbase + M] = 0; v.cflag[cbase + M] = 0; v.cM2[cbase + M] = s.m2[1];
    v.ctail[cbase + M] = s.newpg[pS + pM - 1];
    v.in_req[cbase + M] = 0;
    s.M = M + 1;
    s.a_top = top - from_free + s.nchain;
    s.a_bump = bump + (need - from_free);
    s.nflag -= 1;
    s.did_split = 1;
    v.flist[cbase + pos] = v.flist[cbase + s.nflag];
    count(v, u, 0, 1);
  }
  __syncthreads();
}

template <int DT>
__device__ __forceinline__ void split_cluster(const View& v, int u, int j, int pos, SplitSmem& s) {
  const int tid = threadIdx.x;
  const size_t cbase = (size_t)u * v.Mcap;
  const int m = v.cn[cbase + j] + v.cb[cbase + j];
  if (tid == 0) s.did_split = 0;
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

// ---- small clusters: one wavefront per split ---------------------------------------------------------
// Most clusters that get split hold a few dozen entries at most.  Such a split keeps one wavefront busy, so
// up to four flagged clusters of a unit are split side by side, one per wavefront, with no workgroup barrier
// inside the 2-means: four lanes per member for distances and side tests, lane = coordinate (two each) for sums
// over members.  Same 2-means as split_cluster_impl (seeds, side test with its float64 re-check, rounds, stable
// partition, exact statistics); sums over members are float64 sums of 16-bit values, whose order does not matter.
// What depends on the order of the splits (new cluster ids, page allocation) is done by one thread between the
// two wavefront phases.
// A cluster of up to twice that size (128 entries of a 16-bit type) is split the same way; such a split takes the
// staging rows of two contexts, so only two of them run side by side (a "wide" plan).
constexpr int kWaveSplits = kSplitThreads / 64;
constexpr int kWaveStage = 64 * kStageRow16 * 2;                 // 64 rows of a 16-bit type, 32 of float32
static_assert(32 * kStageRow32 * 4 <= kWaveStage, "float32 rows must fit");
constexpr int kWaveRows = 128;                                   // members of the largest such cluster (16-bit types)
constexpr int kWavePages = kWaveRows / kPageTokens;              // its pages
static_assert(kWavePages <= kInlinePages && kWavePages == 8, "the pages of such a cluster are found without walking its chain");
// Values of the first members (16-byte chunk t = 64k + lane of the member-major array of V rows, k < kVAhead:
// 16 members of a 16-bit type, 8 of float32) are requested together with the keys and wait in registers until
// the children's pages are known.
constexpr int kVAhead = 4;

struct WaveCtx {
  double cA[kHeadDim], cB[kHeadDim];
  alignas(16) float rA[kHeadDim], rB[kHeadDim];
  float d32[kWaveRows];                          // member distances of a seed search
  double m2[2];
  unsigned char side[kWaveRows], perm[kWaveRows], inv[kWaveRows];     // inv[member] = its place in perm
  int chain[kWavePages], newpg[kWavePages + 2];
  int pos[kWaveRows];                            // sequence positions of the members
  int j, m, ok, nS, idM;
  int stage_off;                                 // the staged keys start this many bytes past the context itself
  int pad_[2];
};
// The contexts lie at the front of the split's LDS, the staging rows of all of them behind: context x of a plan
// of small clusters has rows 64x .. 64x + 63, context x = 2, 3 of a wide plan rows 128(x - 2) .. 128(x - 2) + 127.
__device__ __forceinline__ void wave_place_stage(WaveCtx* wc, int x, bool wide) {
  const int row0 = wide ? 128 * (x - 2) : 64 * x;
  wc[x].stage_off = (int)((kWaveSplits - x) * sizeof(WaveCtx)) + row0 * (kWaveStage / 64);
}
__device__ __forceinline__ unsigned char* wave_stage(WaveCtx& c) { return (unsigned char*)&c + c.stage_off; }
__device__ __forceinline__ const unsigned char* wave_stage(const WaveCtx& c) { return (const unsigned char*)&c + c.stage_off; }

__device__ __forceinline__ void wave_sync() {   // LDS written by some lanes of this wavefront, read by others
  asm volatile("" ::: "memory");
  __builtin_amdgcn_wave_barrier();
  asm volatile("" ::: "memory");
}

template <int DT>
__device__ __forceinline__ float wkey(const unsigned char* stage, int i, int d) {
  if constexpr (DT == DYNAKV_F32) return ((const float*)stage)[i * kStageRow32 + d];
  else {
    const uint16_t h = ((const uint16_t*)stage)[i * kStageRow16 + d];
    return DT == DYNAKV_F16 ? f16_to_float(h) : bf16_to_float(h);
  }
}
template <int DT>
__device__ __forceinline__ void wkey8(const unsigned char* stage, int i, int d8, float (&x)[8]) {
  if constexpr (DT == DYNAKV_F32) {
    const f4* p = (const f4*)((const float*)stage + i * kStageRow32 + d8 * 8);
    const f4 a = p[0], b = p[1];
#pragma unroll
    for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
  } else {
    const uint4 w = *(const uint4*)((const uint16_t*)stage + i * kStageRow16 + d8 * 8);
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint16_t h = (uint16_t)(ww[e >> 1] >> ((e & 1) * 16));
      x[e] = DT == DYNAKV_F16 ? f16_to_float(h) : bf16_to_float(h);
    }
  }
}

// Key access in the form quad_sqdist expects.
template <int DT>
struct WaveKeys {
  const unsigned char* stage;
  __device__ void get8(int i, int d8, float (&x)[8]) const { wkey8<DT>(stage, i, d8, x); }
};

// Wavefront arg-max of (value, index), index < 0 = none, equal values to the lowest index; all lanes get it.
// DPP butterfly inside the rows of 16 lanes, row broadcasts across them; lane 63 ends up with the result.
template <int CTRL, int ROWS>
__device__ __forceinline__ void argmax_step(double& val, int& idx) {
  // a lane that the step does not reach sees its own pair
  const int lo = __builtin_amdgcn_update_dpp(__double2loint(val), __double2loint(val), CTRL, ROWS, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(__double2hiint(val), __double2hiint(val), CTRL, ROWS, 0xF, false);
  const int oi = __builtin_amdgcn_update_dpp(idx, idx, CTRL, ROWS, 0xF, false);
  const double ov = __hiloint2double(hi, lo);
  if (oi >= 0 && (idx < 0 || ov > val || (ov == val && oi < idx))) { val = ov; idx = oi; }
}
__device__ __forceinline__ void wave_argmax(double& val, int& idx) {
  argmax_step<kDppXor1, 0xF>(val, idx);
  argmax_step<kDppXor2, 0xF>(val, idx);
  argmax_step<kDppHalfMirror, 0xF>(val, idx);
  argmax_step<kDppMirror, 0xF>(val, idx);
  argmax_step<kDppBcast15, 0xA>(val, idx);
  argmax_step<kDppBcast31, 0xC>(val, idx);
  val = readlane_f64(val, 63);
  idx = __builtin_amdgcn_readlane(idx, 63);
}

// A set of members, wavefront-uniform: bit i of lo = member i, bit i of hi = member 64 + i.
struct MemberSet {
  unsigned long long lo, hi;
};
__device__ __forceinline__ MemberSet first_members(int m) {
  return MemberSet{m >= 64 ? ~0ull : (1ull << m) - 1ull, m <= 64 ? 0ull : m >= 128 ? ~0ull : (1ull << (m - 64)) - 1ull};
}
__device__ __forceinline__ int set_count(MemberSet s) { return __popcll(s.lo) + __popcll(s.hi); }
__device__ __forceinline__ MemberSet set_minus(MemberSet a, MemberSet b) { return MemberSet{a.lo & ~b.lo, a.hi & ~b.hi}; }

// Coordinates 2 lane and 2 lane + 1 of staged member i: one LDS load.
template <int DT>
__device__ __forceinline__ void wpair(const unsigned char* stage, int i, int lane, float& a, float& b) {
  if constexpr (DT == DYNAKV_F32) {
    const float2 x = ((const float2*)((const float*)stage + i * kStageRow32))[lane];
    a = x.x; b = x.y;
  } else {
    const uint32_t w = ((const uint32_t*)((const uint16_t*)stage + i * kStageRow16))[lane];
    a = DT == DYNAKV_F16 ? f16_to_float((uint16_t)w) : bf16_to_float((uint16_t)w);
    b = DT == DYNAKV_F16 ? f16_to_float((uint16_t)(w >> 16)) : bf16_to_float((uint16_t)(w >> 16));
  }
}

// Sums over the members of `set`, in ascending order, of coordinates 2 lane and 2 lane + 1, in float64 (sums of up
// to 128 values of a 16-bit type: exact for float16, and for bfloat16 unless the values of one coordinate span
// more than 2^45).  Eight loads per round trip to LDS; the set is walked with scalar instructions.
template <int DT>
__device__ __forceinline__ void wave_set_sums(const unsigned char* stage, MemberSet set, int lane, double& s0, double& s1) {
  s0 = 0.0; s1 = 0.0;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    unsigned long long mk = half ? set.hi : set.lo;
    while (mk) {
      float x0[8], x1[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const bool in = mk != 0;
        const int i = in ? 64 * half + (int)__builtin_ctzll(mk) : 0;     // member 0 always exists
        mk &= mk - 1;
        float a, b;
        wpair<DT>(stage, i, lane, a, b);
        x0[k] = in ? a : 0.f; x1[k] = in ? b : 0.f;
      }
      asm volatile("" ::: "memory");
#pragma unroll
      for (int k = 0; k < 8; ++k) { s0 += (double)x0[k]; s1 += (double)x1[k]; }
    }
  }
}

// Squared distance of member i to a centre whose coordinates 32 q .. 32 q + 31 are in cr, by the four lanes of a
// quad; every lane gets the total.  Differences, squares and sums in float32: a difference is off by 2^-24 of itself,
// the total by less than 2^-18 of itself.
template <class K>
__device__ __forceinline__ float quad_sqdist32(const K& ks, int i, int q, const float (&cr)[32]) {
  float acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float x[8];
    ks.get8(i, q * 4 + k, x);
    float a = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float t = x[e] - cr[k * 8 + e];
      a = fmaf(t, t, a);
    }
    acc[k] = a;
  }
  float s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), kDppXor1, 0xF, 0xF, false));
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), kDppXor2, 0xF, 0xF, false));
  return s;
}
// This lane's 32 coordinates (32 q ..) of a float32 vector in LDS.
__device__ __forceinline__ void load_quarter(const float* r, int q, float (&fr)[32]) {
#pragma unroll
  for (int e = 0; e < 32; e += 4) {
    const f4 x = *(const f4*)(r + q * 32 + e);
    fr[e] = x[0]; fr[e + 1] = x[1]; fr[e + 2] = x[2]; fr[e + 3] = x[3];
  }
}

// The member farthest from a centre (the lowest index among equals), by one wavefront.  The distances are first
// taken in float32 against the centre rounded to float32 (c.rA); the members within the rounding bound of the
// largest, if there are several, are then compared in float64 against the centre itself (c0, c1: its coordinates
// 2 lane and 2 lane + 1).  cnorm: the centre's norm if rounding it to float32 changed it, else 0.  dub: an upper
// bound of that largest squared distance (the exact value after a float64 comparison).
template <int DT>
__device__ __forceinline__ int wave_farthest(const WaveKeys<DT>& ks, const unsigned char* stage, WaveCtx& c, int m,
                                             double c0, double c1, float cnorm, double& dub) {
  const int lane = threadIdx.x & 63, grp = lane >> 2, kb = lane & 3;
  float cr[32];
  load_quarter(c.rA, kb, cr);
  float fm = -1.f;
  for (int base = 0; base < m; base += 16) {
    const int i = base + grp;
    const float d = quad_sqdist32(ks, min(i, m - 1), kb, cr);
    if (kb == 0 && i < m) { c.d32[i] = d; fm = fmaxf(fm, d); }
  }
  const float top = __int_as_float(wave_max(__float_as_int(fm)));       // distances are >= 0: ordered like their bits
  wave_sync();
  // rounding the centre moves a difference by 2^-24 |centre|, hence the distance by 2^-23 |centre| sqrt(distance)
  const float eps = 2.4e-7f * cnorm * sqrtf(top) + 3.1e-5f * top;
  const float thr = top - 2.f * eps;
  MemberSet cand;
  cand.lo = __ballot(lane < m && c.d32[lane] >= thr);
  cand.hi = m > 64 ? __ballot(lane + 64 < m && c.d32[lane + 64] >= thr) : 0ull;
  if (set_count(cand) == 1) {
    dub = (double)(top + eps);
    return cand.lo ? (int)__builtin_ctzll(cand.lo) : 64 + (int)__builtin_ctzll(cand.hi);
  }
  int best = -1;
  double bv = -1.0;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    unsigned long long mk = half ? cand.hi : cand.lo;
    while (mk) {
      const int i = 64 * half + (int)__builtin_ctzll(mk);
      mk &= mk - 1;
      float a, b;
      wpair<DT>(stage, i, lane, a, b);
      const double d0 = (double)a - c0, d1 = (double)b - c1;
      const double d = wave_sum_f64(fma(d0, d0, d1 * d1));
      if (d > bv) { bv = d; best = i; }
    }
  }
  dub = bv;
  return best;
}

// The same sums for a large set: the four rows of 16 lanes take every fourth member each, a lane adding up the
// eight coordinates of its 16-byte chunk (one LDS load per member and lane); the rows' parts are then added and
// handed to the lanes that own the coordinates through c.cB (which must be free).
template <int DT>
__device__ __forceinline__ void wave_set_sums_rows(const unsigned char* stage, WaveCtx& c, MemberSet set, int m, int lane,
                                                   double& s0, double& s1) {
  const int r = lane >> 4, ch = lane & 15;
  double acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.0;
#pragma unroll 2
  for (int i = r; i < m; i += 4) {
    const bool in = (((i < 64 ? set.lo : set.hi) >> (i & 63)) & 1ull) != 0;
    float x[8];
    wkey8<DT>(stage, i, ch, x);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += in ? (double)x[e] : 0.0;
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    acc[e] += __shfl_xor(acc[e], 16);
    acc[e] += __shfl_xor(acc[e], 32);
  }
  if (r == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) c.cB[8 * ch + e] = acc[e];
  }
  wave_sync();
  s0 = c.cB[2 * lane]; s1 = c.cB[2 * lane + 1];
  wave_sync();
}
// Either way, by the size of the set.
template <int DT>
__device__ __forceinline__ void wave_sums_of(const unsigned char* stage, WaveCtx& c, MemberSet set, int m, int lane,
                                             double& s0, double& s1) {
  if (set_count(set) > 48) wave_set_sums_rows<DT>(stage, c, set, m, lane, s0, s1);
  else wave_set_sums<DT>(stage, set, lane, s0, s1);
}

// quad_side with the float32 weights of coordinates 32 q .. 32 q + 31 already in registers (wr).
template <class K>
__device__ __forceinline__ unsigned char quad_side_reg(const K& ks, int i, int q, const float (&wr)[32], const double* wd,
                                                       double t, float eps) {
  float x[4][8];
#pragma unroll
  for (int k = 0; k < 4; ++k) ks.get8(i, q * 4 + k, x[k]);
  float part[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float a = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) a = fmaf(x[k][e], wr[k * 8 + e], a);
    part[k] = a;
  }
  float s = (part[0] + part[1]) + (part[2] + part[3]);
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), kDppXor1, 0xF, 0xF, false));
  s += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), kDppXor2, 0xF, 0xF, false));
  const float tf = (float)t;
  if (fabsf(s - tf) > eps) return s <= tf ? 0 : 1;            // uniform over the quad
  double sd = 0.0;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) sd = fma((double)x[k][e], wd[(q * 4 + k) * 8 + e], sd);
  sd += dpp_f64<kDppXor1, 0xF>(sd);
  sd += dpp_f64<kDppXor2, 0xF>(sd);
  return sd <= t ? 0 : 1;
}

// One wavefront decides one split: stages the keys (c.chain lists their pages), 2-means, stable partition, exact
// statistics of the children (of the unsplit cluster if the 2-means finds nothing to split).  Sets c.ok, c.nS,
// c.perm, c.inv, c.pos, the float32 means c.rA / c.rB and the M2 about them, c.m2.
// Lanes stand for coordinates (2 lane, 2 lane + 1) in sums over members, for quarter members (four lanes each) in
// distances and side tests; the sides of a round are two 64-bit sets, and the sum of side A follows the members
// that changed side instead of being formed anew.
template <int DT, bool AHEAD>
__device__ inline void wave_split_decide(const View& v, int u, WaveCtx& c, uint4 (&vahead)[kVAhead]) {
  const int lane = threadIdx.x & 63;
  constexpr int kEs = DT == DYNAKV_F32 ? 4 : 2;
  constexpr int kChunks = kHeadDim * kEs / 16;
  constexpr int kRowBytes = (DT == DYNAKV_F32 ? kStageRow32 : kStageRow16) * kEs;
  constexpr int kAhead = 16;                               // key loads in flight per lane
  const char* const pool = v.pages + (size_t)u * v.Pcap * ((size_t)kPageElems * kEs);
  const int m = c.m;
  unsigned char* const stage = wave_stage(c);
  const int total = m * kChunks;
  for (int t0 = 0; t0 < total; t0 += kAhead * 64) {
    f4 w[kAhead];                                          // (a plain vector type: these stay in registers)
#pragma unroll
    for (int k = 0; k < kAhead; ++k) {
      const int t = min(t0 + k * 64 + lane, total - 1);
      const int i = t / kChunks, ch = t % kChunks;
      const size_t off = (size_t)(DT == DYNAKV_F32 ? k_index32(i & 15, 4 * ch) : k_index16(i & 15, 8 * ch)) * kEs;
      w[k] = *(const f4*)(pool + (size_t)c.chain[i >> 4] * (kPageElems * kEs) + off);
    }
    if (t0 == 0) {                                         // the values requested ahead and the positions ride along
#pragma unroll
      for (int k = 0; k < kVAhead; ++k) {
        const int t = k * 64 + lane, i = t / kChunks, ch = t % kChunks;
        vahead[k] = uint4{0, 0, 0, 0};
        if (AHEAD && i < m) {
          const size_t off = (size_t)(DT == DYNAKV_F32 ? v_index32(i & 15, 4 * ch) : v_index16(i & 15, 8 * ch)) * kEs;
          vahead[k] = *(const uint4*)(pool + (size_t)c.chain[i >> 4] * (kPageElems * kEs) + off);
        }
      }
      for (int i = lane; i < m; i += 64) c.pos[i] = v.ppos[((size_t)u * v.Pcap + c.chain[i >> 4]) * kPageTokens + (i & 15)];
    }
#pragma unroll
    for (int k = 0; k < kAhead; ++k) {
      const int t = t0 + k * 64 + lane;
      if (t < total) *(f4*)(stage + (size_t)(t / kChunks) * kRowBytes + (t % kChunks) * 16) = w[k];
    }
  }
  wave_sync();
  const WaveKeys<DT> ks{stage};
  const int grp = lane >> 2, kb = lane & 3;      // four lanes per member in the distance passes
  const MemberSet all = first_members(m);
  double tot0, tot1;
  wave_set_sums_rows<DT>(stage, c, all, m, lane, tot0, tot1);
  double sa0 = tot0, sa1 = tot1;                 // sum of side A
  MemberSet A = all;
  bool can = m >= 2;
  if (can) {
    // seeds: A = member farthest from the mean of all members, B = member farthest from A
    const double mu0 = tot0 / (double)m, mu1 = tot1 / (double)m;
    const double mn2 = wave_sum_f64(mu0 * mu0 + mu1 * mu1);
    c.rA[2 * lane] = (float)mu0; c.rA[2 * lane + 1] = (float)mu1;
    wave_sync();
    double dmax, db;
    const int a = wave_farthest<DT>(ks, stage, c, m, mu0, mu1, (float)sqrt(mn2) * 1.0001f, dmax);
    float fa0, fa1;
    wpair<DT>(stage, a, lane, fa0, fa1);
    double ca0 = (double)fa0, ca1 = (double)fa1;                             // seed A
    c.rA[2 * lane] = fa0; c.rA[2 * lane + 1] = fa1;
    wave_sync();
    const int b = wave_farthest<DT>(ks, stage, c, m, ca0, ca1, 0.f, db);
    can = db > 0.0;                          // false: all members identical
    if (can) {
      // every member lies within sqrt(dmax) of the mean, and so does every centre (a mean of members)
      const float spread = (float)sqrt(dmax) * 1.0001f;
      const float xmax = spread + (float)sqrt(mn2) * 1.0001f;
      float fb0, fb1;
      wpair<DT>(stage, b, lane, fb0, fb1);
      double cb0 = (double)fb0, cb1 = (double)fb1;                           // seed B
      bool first = true;
      for (int it = 0; it < 16; ++it) {
        // w = cB - cA into c.cA (float64) and c.rA (float32), t = (|cB|^2 - |cA|^2) / 2
        const double w0 = cb0 - ca0, w1 = cb1 - ca1;
        const double t = wave_sum_f64(0.5 * ((cb0 * cb0 - ca0 * ca0) + (cb1 * cb1 - ca1 * ca1)));
        c.cA[2 * lane] = w0; c.cA[2 * lane + 1] = w1;
        c.rA[2 * lane] = (float)w0; c.rA[2 * lane + 1] = (float)w1;
        wave_sync();
        const float eps = side_eps(xmax, 2.f * spread, t);
        float wr[32];
        load_quarter(c.rA, kb, wr);
        for (int base = 0; base < m; base += 16) {
          const int i = base + grp;
          const unsigned char ns = quad_side_reg(ks, min(i, m - 1), kb, wr, c.cA, t, eps);
          if (kb == 0 && i < m) c.side[i] = ns;
        }
        wave_sync();
        MemberSet nw;
        nw.lo = __ballot(lane < m && c.side[lane] == 0);
        nw.hi = m > 64 ? __ballot(lane + 64 < m && c.side[lane + 64] == 0) : 0ull;
        if (!first && nw.lo == A.lo && nw.hi == A.hi) break;          // no member moved
        const int nA = set_count(nw);
        if (nA == 0 || nA == m) { can = false; break; }
        // the sum of side A: formed from the smaller side in the first round, then corrected by the members that
        // moved; side B is what is left of the total
        double j0, j1, l0, l1;
        if (first) {
          if (2 * nA <= m) wave_sums_of<DT>(stage, c, nw, m, lane, sa0, sa1);
          else {
            wave_sums_of<DT>(stage, c, set_minus(all, nw), m, lane, l0, l1);
            sa0 = tot0 - l0; sa1 = tot1 - l1;
          }
        } else {
          wave_sums_of<DT>(stage, c, set_minus(nw, A), m, lane, j0, j1);
          wave_sums_of<DT>(stage, c, set_minus(A, nw), m, lane, l0, l1);
          sa0 += j0 - l0; sa1 += j1 - l1;
        }
        A = nw; first = false;
        const double ia = 1.0 / (double)nA, ib = 1.0 / (double)(m - nA);     // (centres of a round: one rounding more is harmless)
        ca0 = sa0 * ia; ca1 = sa1 * ia;
        cb0 = (tot0 - sa0) * ib; cb1 = (tot1 - sa1) * ib;
      }
    }
  }
  // stable partition: the child that holds the earliest entry comes first and keeps the id
  MemberSet S = all;
  if (can) S = (A.lo & 1ull) ? A : set_minus(all, A);
  const int n0 = __popcll(S.lo), nS = n0 + __popcll(S.hi), nM = m - nS;
  {
    const unsigned long long below = (1ull << lane) - 1ull;
    if (lane < m) {
      const int before = __popcll(S.lo & below);
      const int q = (S.lo >> lane) & 1ull ? before : nS + lane - before;
      c.perm[q] = (unsigned char)lane;
      c.inv[lane] = (unsigned char)q;
    }
    if (lane + 64 < m) {
      const int before = n0 + __popcll(S.hi & below);
      const int q = (S.hi >> lane) & 1ull ? before : nS + (lane + 64) - before;
      c.perm[q] = (unsigned char)(lane + 64);
      c.inv[lane + 64] = (unsigned char)q;
    }
  }
  if (lane == 0) { c.ok = can ? 1 : 0; c.nS = nS; }
  // statistics: float32 means of the children, then M2 about those means (differences in float32, off by 2^-24 of
  // themselves; sums of 32 squares in float32, the rest in float64)
  double sS0 = tot0, sS1 = tot1;
  if (can && (A.lo & 1ull)) { sS0 = sa0; sS1 = sa1; }
  else if (can) { sS0 = tot0 - sa0; sS1 = tot1 - sa1; }
  c.rA[2 * lane] = (float)(sS0 / (double)nS); c.rA[2 * lane + 1] = (float)(sS1 / (double)nS);
  if (can) {
    c.rB[2 * lane] = (float)((tot0 - sS0) / (double)nM); c.rB[2 * lane + 1] = (float)((tot1 - sS1) / (double)nM);
  }
  wave_sync();
  double acc[2] = {0.0, 0.0};
#pragma unroll
  for (int child = 0; child < 2; ++child) {
    const int q0 = child ? nS : 0, q1 = child ? m : nS;
    if (q1 <= q0) continue;
    float fr[32];
    load_quarter(child ? c.rB : c.rA, kb, fr);
    for (int base = q0; base < q1; base += 16) {
      const int q = base + grp;
      const float dv = quad_sqdist32(ks, c.perm[min(q, q1 - 1)], kb, fr);
      if (kb == 0 && q < q1) acc[child] += (double)dv;
    }
  }
  const double m2S = wave_sum_f64(acc[0]), m2M = wave_sum_f64(acc[1]);
  if (lane == 0) { c.m2[0] = m2S; c.m2[1] = m2M; }
  wave_sync();
}

// Last phase, one wavefront, once the children's id and pages are assigned: pages, centroids and records.  With
// c.ok == 0 the cluster is only unflagged, with exact statistics.  wave_split_decide has run on c.
template <int DT>
__device__ inline void wave_split_commit(const View& v, int u, WaveCtx& c, const uint4 (&vahead)[kVAhead],
                                         bool ahead) {
  const int lane = threadIdx.x & 63;
  const size_t cbase = (size_t)u * v.Mcap;
  constexpr int kEs = DT == DYNAKV_F32 ? 4 : 2;
  constexpr int kChunks = kHeadDim * kEs / 16;
  constexpr int kRowBytes = (DT == DYNAKV_F32 ? kStageRow32 : kStageRow16) * kEs;
  constexpr size_t kPageBytes = (size_t)kPageElems * kEs;
  char* const pool = v.pages + (size_t)u * v.Pcap * kPageBytes;
  const int m = c.m, j = c.j, nS = c.nS, nM = m - nS, idM = c.ok ? c.idM : -1;
  const int pS = (nS + kPageTokens - 1) / kPageTokens, pM = (nM + kPageTokens - 1) / kPageTokens, need = pS + pM;
  const unsigned char* const stage = wave_stage(c);
  if (c.ok) {
    if (lane < need) v.pnext[(size_t)u * v.Pcap + c.newpg[lane]] = (lane == pS - 1 || lane == need - 1) ? -1 : c.newpg[lane + 1];
    for (int t = lane; t < m * kChunks; t += 64) {
      const int q = t / kChunks, ch = t % kChunks;
      const int i = c.perm[q];
      const int r = q < nS ? q : q - nS;
      const int dpage = c.newpg[(q < nS ? 0 : pS) + (r >> 4)];
      const size_t off = (size_t)(DT == DYNAKV_F32 ? k_index32(r & 15, 4 * ch) : k_index16(r & 15, 8 * ch)) * kEs;
      *(uint4*)(pool + (size_t)dpage * kPageBytes + off) = *(const uint4*)(stage + (size_t)i * kRowBytes + ch * 16);
    }
    // values chunk by chunk like the keys, straight from their old pages: first the chunks requested ahead
    auto vchunk = [](int slot, int ch) -> size_t {
      return (size_t)(DT == DYNAKV_F32 ? v_index32(slot, 4 * ch) : v_index16(slot, 8 * ch)) * kEs;
    };
    auto vdest = [&](int i, int ch) -> char* {
      const int q = c.inv[i];
      const int r = q < nS ? q : q - nS;
      return (char*)pool + (size_t)c.newpg[(q < nS ? 0 : pS) + (r >> 4)] * kPageBytes + vchunk(r & 15, ch);
    };
    if (ahead) {
#pragma unroll
      for (int k = 0; k < kVAhead; ++k) {
        const int t = k * 64 + lane, i = t / kChunks;
        if (i < m) *(uint4*)vdest(i, t % kChunks) = vahead[k];
      }
    }
    // then the members past those (all, if nothing was requested ahead), sixteen loads in flight per lane
    constexpr int kVFlight = 16;
    for (int t0 = ahead ? kVAhead * 64 : 0; t0 < m * kChunks; t0 += kVFlight * 64) {
      f4 w[kVFlight];
#pragma unroll
      for (int k = 0; k < kVFlight; ++k) {
        const int t = min(t0 + k * 64 + lane, m * kChunks - 1), i = t / kChunks;
        w[k] = *(const f4*)(pool + (size_t)c.chain[i >> 4] * kPageBytes + vchunk(i & 15, t % kChunks));
      }
#pragma unroll
      for (int k = 0; k < kVFlight; ++k) {
        const int t = t0 + k * 64 + lane;
        if (t < m * kChunks) *(f4*)vdest(t / kChunks, t % kChunks) = w[k];
      }
    }
    for (int i = lane; i < m; i += 64) {
      const int q = c.inv[i];
      const int r = q < nS ? q : q - nS;
      const int dpage = c.newpg[(q < nS ? 0 : pS) + (r >> 4)];
      v.ppos[((size_t)u * v.Pcap + dpage) * kPageTokens + (r & 15)] = c.pos[i];
    }
  }
  store_centroid(v, u, j, lane, c.rA[lane]); store_centroid(v, u, j, lane + 64, c.rA[lane + 64]);
  if (idM >= 0) { store_centroid(v, u, idM, lane, c.rB[lane]); store_centroid(v, u, idM, lane + 64, c.rB[lane + 64]); }
  if (c.ok && lane < kInlinePages) {
    v.cpg[(cbase + j) * kInlinePages + lane] = lane < pS ? c.newpg[lane] : -1;
    v.cpg[(cbase + idM) * kInlinePages + lane] = lane < pM ? c.newpg[pS + lane] : -1;
  }
  if (lane == 0) {
    v.cn[cbase + j] = nS; v.csz[cbase + j] = nS; v.cb[cbase + j] = 0; v.cflag[cbase + j] = 0; v.cM2[cbase + j] = c.m2[0];
    if (c.ok) {
      v.ctail[cbase + j] = c.newpg[pS - 1];
      v.cn[cbase + idM] = nM; v.csz[cbase + idM] = nM; v.cb[cbase + idM] = 0; v.cflag[cbase + idM] = 0; v.cM2[cbase + idM] = c.m2[1];
      v.ctail[cbase + idM] = c.newpg[pS + pM - 1];
      v.in_req[cbase + idM] = 0;
    }
  }
}

// Plan of one unit's splits, made from the list of its flagged clusters (at most 64 of them).
constexpr int kFreeAhead = 24;
struct SplitPlan {
  int id[64], req[64], cb[64], m[64];   // the flagged clusters
  alignas(16) int pg[64][kWavePages];   // their first pages
  int cand[64];                          // positions in the list, in the order of the splits
  int n_cand, forced, fast;
  int wide;                              // some cluster of the plan needs two members per lane: two splits at a time
  int M, top, bump;                      // the unit's counters while the plan is carried out
  int fl[kFreeAhead], fl_base;           // top of the free-page stack, read ahead: fl[k] = entry fl_base - 1 - k
};

// LDS of one unit's splits: `raw` holds either the workgroup-wide split or four wavefront splits.
constexpr size_t kWaveRaw = kWaveSplits * (sizeof(WaveCtx) + kWaveStage);
constexpr size_t kSplitRaw = sizeof(SplitSmem) > kWaveRaw ? sizeof(SplitSmem) : kWaveRaw;
static_assert(sizeof(WaveCtx) % 16 == 0, "the staging rows behind the contexts are 16-byte aligned");
struct SplitWork {
  SplitPlan pl;
  long long s_tot;
  int s_min;
  int nf0, M0, npre;                     // left by plan_finish: flagged clusters, clusters, splits decided ahead
  int ready;                             // set (release) once the plan is in place, for wavefronts that do not share a
                                         // barrier with the one that made it
  int flagged0[64], nflag0, top0;        // for plan_fetch_early: the flagged list and the free stack before the append
};
// Candidate k of a round of wavefront splits is handled by wavefront k and held in context ctx_of(k): the
// contexts of the first candidates lie at the far end of `raw`, clear of what a caller of split_predecide may
// still be using at the front.
__device__ __forceinline__ int ctx_of(int k) { return kWaveSplits - 1 - k; }

// What the plan needs about one flagged cluster; id < 0: no cluster.
struct PlanEntry {
  int id, req, cb, m;
};
// Fetches it for flagged cluster `c` (slot i of the plan), into the plan and for the calling lane.
__device__ __forceinline__ PlanEntry plan_fetch(const View& v, size_t cbase, SplitPlan& pl, int i, int c) {
  const int b = v.cb[cbase + c];
  const int4 pg = *(const int4*)&v.cpg[(cbase + c) * kInlinePages];
  const int4 pg2 = *(const int4*)&v.cpg[(cbase + c) * kInlinePages + 4];
  const PlanEntry e{c, v.in_req[cbase + c], b, v.cn[cbase + c] + b};
  pl.id[i] = e.id; pl.req[i] = e.req; pl.cb[i] = e.cb; pl.m[i] = e.m;
  *(int4*)&pl.pg[i][0] = pg; *(int4*)&pl.pg[i][4] = pg2;
  return e;
}
// Everything the page allocation will need, requested in the same round trip: entry k of the read-ahead.
__device__ __forceinline__ void plan_fetch_pages(const View& v, int u, SplitPlan& pl, int k, int top, int M0) {
  if (k < top) pl.fl[k] = v.freelist[(size_t)u * v.Pcap + top - 1 - k];
  if (k == 0) { pl.M = M0; pl.top = top; pl.bump = v.bump[u]; pl.fl_base = top; }
}

// The order of the unit's splits, by one whole wavefront: lane i < nf0 <= 64 brings flagged cluster i (e.id < 0 in
// the other lanes); pl.M, pl.top and pl.bump are in place.  Delayed splits first: flagged clusters of the active
// set (all flagged ones if nothing is buffered) in ascending id; then, if the remaining buffers hold B_max
// entries, the fullest of them (lowest id among equals).
template <int DT>
__device__ inline void plan_splits(const View& v, SplitPlan& pl, const PlanEntry& e) {
  const int lane = threadIdx.x & 63;
  const bool have = e.id >= 0;
  const bool delayed = have && (v.Bmax == 0 || e.req != 0);
  const unsigned long long dmask = __ballot(delayed);
  int rank = 0;
  for (unsigned long long mm = dmask; mm; mm &= mm - 1) {          // ids are distinct: rank = smaller ids
    const int other = __shfl(e.id, __ffsll((long long)mm) - 1);
    rank += other < e.id ? 1 : 0;
  }
  if (delayed) pl.cand[rank] = lane;
  int nc = __popcll(dmask), forced = 0, fl = -1;
  if (v.Bmax > 0) {
    const bool rest = have && !delayed;
    const int total = wave_sum(rest ? e.cb : 0);
    const int bcb = wave_max(rest ? e.cb : -1);                                  // the fullest buffer ...
    const int bid = wave_min(rest && e.cb == bcb ? e.id : 0x7ffffffe);           // ... of the lowest id among equals
    const unsigned long long who = __ballot(rest && e.cb == bcb && e.id == bid);
    const int bl = who ? __ffsll((long long)who) - 1 : 0;
    if (bcb >= 0 && total >= v.Bmax) {
      if (lane == 0) pl.cand[nc] = bl;
      fl = bl; ++nc; forced = 1;
    }
  }
  // the wavefront path takes the plan if every cluster is small and no capacity limit can be hit
  constexpr int kSmall = DT == DYNAKV_F32 ? 32 : 64;                 // one member per lane; twice that: a wide plan
  const bool isc = delayed || lane == fl;
  const bool small = __ballot(isc && e.m > 2 * kSmall) == 0;
  const bool wide = __ballot(isc && e.m > kSmall) != 0;
  int pages = isc ? (e.m + kPageTokens - 1) / kPageTokens + 1 : 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) pages += __shfl_xor(pages, o);
  if (lane == 0) {
    pl.n_cand = nc; pl.forced = forced; pl.wide = wide ? 1 : 0;
    pl.fast = small && pl.M + nc <= v.Mcap && pages <= pl.top + (v.Pcap - pl.bump);
  }
}

// Hands candidate `at` of the plan to context c (one wavefront).
__device__ __forceinline__ void wave_take(const SplitPlan& pl, int at, WaveCtx* wc, int x, int lane) {
  WaveCtx& c = wc[x];
  if (lane == 0) { c.j = pl.id[at]; c.m = pl.m[at]; wave_place_stage(wc, x, pl.wide != 0); }
  if (lane < kWavePages) c.chain[lane] = pl.pg[at][lane];
  wave_sync();
}

// ---- head start for split_unit inside a kernel that has just selected the active set and appended a token ----
// The plan's inputs are requested before the append is committed (plan_fetch_early, first wavefront, after the
// selection), corrected for what the append changed and turned into the plan right after it (plan_finish); the
// first splits of the plan can then be decided (split_predecide, one wavefront each) while the rest
// of the workgroup is busy elsewhere: deciding only reads the index.
struct PlanEarly {
  int id, req, cb, cn;     // lane i < nflag0: flagged cluster i; lane nflag0: the cluster the append may flag
  int fl0, bump0;          // free-page stack entry top0 - 1 - lane; bump pointer
  int4 pg, pg2;
};
// flagged0: entry `lane` of the flagged list, nflag0 its length, top0 the height of the free-page stack, all as
// they are before the append; ja: the cluster the append goes to (< 0: no append).
// selbits: the active set of the selection that has just run, one bit per cluster (LDS).
__device__ __forceinline__ PlanEarly plan_fetch_early(const View& v, int u, int flagged0, int nflag0, int top0, int ja,
                                                      int lane, const unsigned* selbits) {
  const size_t cbase = (size_t)u * v.Mcap;
  PlanEarly e{-1, 0, 0, 0, 0, 0, int4{-1, -1, -1, -1}, int4{-1, -1, -1, -1}};
  const int c = lane < nflag0 ? flagged0 : lane == nflag0 ? ja : -1;
  if (c >= 0 && nflag0 <= 64) {
    e.id = c; e.req = (selbits[c >> 5] >> (c & 31)) & 1u; e.cb = v.cb[cbase + c]; e.cn = v.cn[cbase + c];
    e.pg = *(const int4*)&v.cpg[(cbase + c) * kInlinePages];
    e.pg2 = *(const int4*)&v.cpg[(cbase + c) * kInlinePages + 4];
  }
  if (lane <= kFreeAhead && lane < top0) e.fl0 = v.freelist[(size_t)u * v.Pcap + top0 - 1 - lane];
  e.bump0 = v.bump[u];
  return e;
}
// First wavefront, after the append (a: its record, null if there was none) and a barrier.  Leaves the plan in
// wk.pl and wk.nf0 / M0 / npre (npre <= max_pre = splits to decide ahead).
template <int DT>
__device__ inline void plan_finish(const View& v, SplitWork& wk, PlanEarly e, int nflag0, int top0, int M, int ja,
                                   const AppendSmem* a, int max_pre) {
  SplitPlan& pl = wk.pl;
  const int lane = threadIdx.x & 63;
  int nf = nflag0, top = top0, bump = e.bump0;
  if (a && a->ok) {
    nf = a->nflag1; top = a->top1; bump = a->bump1;
    const int sz = a->cn + a->cb;                        // entries of cluster ja before the append
    const bool newflag = nf > nflag0;
    if (newflag ? lane == nflag0 : (lane < nflag0 && e.id == ja)) {
      e.cb = newflag ? 1 : e.cb + 1;                     // the token went to the buffer of a flagged cluster
      if (a->slot == 0) {                                // and opened a page
        const int k = sz / kPageTokens;
        if (k == 0) e.pg.x = a->page;
        else if (k == 1) e.pg.y = a->page;
        else if (k == 2) e.pg.z = a->page;
        else if (k == 3) e.pg.w = a->page;
        else if (k == 4) e.pg2.x = a->page;
        else if (k == 5) e.pg2.y = a->page;
        else if (k == 6) e.pg2.z = a->page;
        else if (k == 7) e.pg2.w = a->page;
      }
    }
  }
  if (lane >= nf) e.id = -1;
  const int fl = __shfl(e.fl0, min(lane + (top0 - top), 63));     // the append took at most the top page
  if (lane == 0) {
    wk.nf0 = nf; wk.M0 = M; wk.npre = 0;
    pl.fast = 0; pl.M = M; pl.top = top; pl.bump = bump; pl.fl_base = top;
  }
  if (nf == 0 || nf > 64) return;
  if (lane < kFreeAhead && lane < top) pl.fl[lane] = fl;
  if (e.id >= 0) {
    pl.id[lane] = e.id; pl.req[lane] = e.req; pl.cb[lane] = e.cb; pl.m[lane] = e.cn + e.cb;
    *(int4*)&pl.pg[lane][0] = e.pg; *(int4*)&pl.pg[lane][4] = e.pg2;
  }
  wave_sync();
  plan_splits<DT>(v, pl, PlanEntry{e.id, e.req, e.cb, e.cn + e.cb});
  wave_sync();
  if (lane == 0) wk.npre = pl.fast ? min(pl.n_cand, min(max_pre, pl.wide ? kWaveSplits / 2 : kWaveSplits)) : 0;
}
// Wavefront k < wk.npre decides split k of the plan and computes the children's statistics, into context
// ctx_of(k) of `raw`; pre_v: the values requested ahead, for the same wavefront to hand to split_unit.
template <int DT>
__device__ inline void split_predecide(const View& v, int u, unsigned char* raw, const SplitWork& wk, int k,
                                       uint4 (&pre_v)[kVAhead]) {
  WaveCtx& c = ((WaveCtx*)raw)[ctx_of(k)];
  // the split is the longest chain of dependent steps of its unit: it goes ahead of the wavefront that streams pages
  // on the same SIMD (the tiles that one does not take meanwhile go to the other wavefronts)
  __builtin_amdgcn_s_setprio(3);
  wave_take(wk.pl, wk.pl.cand[k], (WaveCtx*)raw, ctx_of(k), threadIdx.x & 63);
  wave_split_decide<DT, true>(v, u, c, pre_v);
  __builtin_amdgcn_s_setprio(0);
}

// One thread: ids and pages for the decided splits base .. base + n - 1 of the plan (contexts ctx_of(0 .. n-1)),
// in the order of the plan.
__device__ inline void split_assign(const View& v, int u, WaveCtx* wc, SplitPlan& pl, int n) {
  for (int w = 0; w < n; ++w) {
    WaveCtx& cw = wc[ctx_of(w)];
    if (!cw.ok) continue;
    cw.idM = pl.M++;
    const int need = (cw.nS + kPageTokens - 1) / kPageTokens + (cw.m - cw.nS + kPageTokens - 1) / kPageTokens;
    const int from_free = min(need, pl.top);
    for (int k = 0; k < need; ++k) {
      const int ra = pl.fl_base - (pl.top - k);          // pl.fl holds the stack as it was at fl_base
      cw.newpg[k] = k >= from_free ? pl.bump + (k - from_free)
                    : (ra >= 0 && ra < kFreeAhead) ? pl.fl[ra]
                                                    : v.freelist[(size_t)u * v.Pcap + pl.top - 1 - k];
    }
    pl.top -= from_free;
    pl.bump += need - from_free;
  }
}
// One thread, once the n splits are committed and nothing reads the parents' pages any more: recycles them.
// base: place of the first of them in the plan (a forced split is the plan's last entry and is counted as forced
// only if it was carried out).
__device__ inline void split_recycle(const View& v, int u, const WaveCtx* wc, SplitPlan& pl, int n, int base) {
  for (int w = 0; w < n; ++w) {
    const WaveCtx& cw = wc[ctx_of(w)];
    count(v, u, (cw.ok ? 0 : 1), 1);
    if (cw.ok && pl.forced && base + w == pl.n_cand - 1) count(v, u, 2, 1);
    if (!cw.ok) continue;
    const int npg = (cw.m + kPageTokens - 1) / kPageTokens;
    for (int k = 0; k < npg; ++k) v.freelist[(size_t)u * v.Pcap + pl.top++] = cw.chain[k];
    pl.fl_base = -(1 << 30);         // the stack has changed: what was read ahead no longer applies
  }
}

// All splits of unit u that are due (Algorithm 1, decode block: delayed splits, then the forced one), by the
// first kSplitThreads threads of the workgroup; no other thread of the workgroup may still be running.
// raw: kSplitRaw bytes of LDS, 16-byte aligned.  prepared: plan_finish and split_predecide have run and the
// caller has assigned (split_assign) and committed (wave_split_commit) the wk.npre splits decided ahead, with a
// barrier since; their parents' pages are still to be recycled.
template <int DT>
__device__ __forceinline__ void split_unit(const View& v, int u, unsigned char* raw, SplitWork& wk, bool prepared) {
  constexpr int NT = kSplitThreads;
  SplitPlan& pl = wk.pl;
  int& s_min = wk.s_min;
  long long& s_tot = wk.s_tot;
  SplitSmem& s = *(SplitSmem*)raw;
  WaveCtx* const wc = (WaveCtx*)raw;
  const int tid = threadIdx.x;
  const size_t cbase = (size_t)u * v.Mcap;
  int M0, nf0, npre = 0;
  if (prepared) {
    M0 = wk.M0; nf0 = wk.nf0; npre = wk.npre;
    if (nf0 == 0) return;
  } else {
    // requested together with the flag count, so that the plan below starts one round trip earlier
    const int c_ahead = tid < min(64, v.Mcap) ? v.flist[cbase + tid] : 0;
    const int top_ahead = v.free_top[u];
    M0 = v.M[u];
    nf0 = v.nflag[u];
    if (nf0 == 0) return;
    if (nf0 <= 64) {
      PlanEntry e{-1, 0, 0, 0};
      if (tid < nf0) e = plan_fetch(v, cbase, pl, tid, c_ahead);
      if (tid >= 64 && tid < 64 + kFreeAhead) plan_fetch_pages(v, u, pl, tid - 64, top_ahead, M0);
      __syncthreads();
      if (tid < 64) plan_splits<DT>(v, pl, e);
      __syncthreads();
    }
  }

  // ---- the plan's splits, up to four side by side, one per wavefront
  if (nf0 <= 64) {
    if (pl.fast) {
      const int wave = tid >> 6, lane = tid & 63;
      const int nc = pl.n_cand;
      const int side_by_side = pl.wide ? kWaveSplits / 2 : kWaveSplits;
      if (npre > 0) {                      // committed by the caller
        if (tid == 0) split_recycle(v, u, wc, pl, npre, 0);
        __syncthreads();
      }
      for (int base = npre; base < nc; base += side_by_side) {
        const int mk = base + wave;                    // this wavefront's candidate
        const bool mine = wave < side_by_side && mk < nc;
        const int n = min(side_by_side, nc - base);
        uint4 vahead[kVAhead];
        WaveCtx& c = wc[ctx_of(wave)];
        if (mine) {
          wave_take(pl, pl.cand[mk], wc, ctx_of(wave), lane);
          wave_split_decide<DT, true>(v, u, c, vahead);
        }
        __syncthreads();
        if (tid == 0) split_assign(v, u, wc, pl, n);             // ids and pages, in the order of the splits
        __syncthreads();
        if (mine) wave_split_commit<DT>(v, u, c, vahead, true);
        __syncthreads();
        if (tid == 0) split_recycle(v, u, wc, pl, n, base);      // the parents' pages are recycled only now
        __syncthreads();
      }
      if (tid == 0 && nc > 0) {            // (no split: list and counters are as they were)
        int n = 0;
        for (int k = 0; k < nc; ++k) pl.id[pl.cand[k]] = -1;
        for (int i = 0; i < nf0; ++i)
          if (pl.id[i] >= 0) v.flist[cbase + n++] = pl.id[i];
        v.nflag[u] = n; v.M[u] = pl.M; v.free_top[u] = pl.top; v.bump[u] = pl.bump;
      }
      return;
    }
  }

  // ---- general path: one split at a time by the whole workgroup
  if (tid == 0) { s.M = M0; s.nflag = nf0; s.a_top = v.free_top[u]; s.a_bump = v.bump[u]; }
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
        if (c >= cursor && c < M0 && (v.Bmax == 0 || v.in_req[cbase + c])) atomicMin(&s_min, c);
      }
      __syncthreads();
      if (s_min != 0x7FFFFFFF) j = s_min;
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
        if ((double)b > bv || ((double)b == bv && c < bi)) { bv = (double)b; bi = c; }
      }
      if (tot) atomicAdd((unsigned long long*)&s_tot, (unsigned long long)tot);
      block_argmax(bv, bi, s.sv, s.si);
      const int arg = s.si[0];
      const long long total = s_tot;
      __syncthreads();
      if (!(arg >= 0 && total >= v.Bmax)) break;
      j = arg;
    }
    // the cluster's place in the list of flagged clusters
    if (tid == 0) s_min = -1;
    __syncthreads();
    for (int i = tid; i < nf; i += NT)
      if (v.flist[cbase + i] == j) s_min = i;
    __syncthreads();
    pos = s_min;
    __syncthreads();
    split_cluster<DT>(v, u, j, pos, s);
    if (forced_done && tid == 0 && s.did_split) count(v, u, 2, 1);     // a forced split counts once carried out
    __syncthreads();
    if (forced_done) break;
  }
  __syncthreads();
  if (tid == 0) { v.M[u] = s.M; v.nflag[u] = s.nflag; v.free_top[u] = s.a_top; v.bump[u] = s.a_bump; }
}

}  // namespace

}  // namespace dynakv
