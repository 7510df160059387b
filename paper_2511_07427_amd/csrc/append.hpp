// The part of an append that follows the nearest-cluster search (Algorithm 1, decode block; UpdateVar of
// Section 4.2): shared by the stand-alone append kernel and by the retrieval kernel that finds the nearest
// cluster during its own pass over the centroid table.
#pragma once
#include "common.hpp"

namespace dynakv {

struct AppendSmem {
  double kd[kHeadDim];       // the new key, filled (and synchronised) by the caller
  double delta[kHeadDim], r1[kHeadDim];
  double bs[16];             // block sums of the M2 increment
  double m2, tau;
  int cn, cb, ctail, cflag, nflag, free_top, bump, free_page;
  int ok, commit, page, slot;
  int nflag1, top1, bump1;   // the unit's flag count and allocator state as the append leaves them
};

// What one thread fetches for an append: thread d < 128 coordinate d of the centroid, threads 128..136 one field
// each of the cluster's record or of the unit's allocator state.  All of it in one round trip to memory.
struct AppendFetch {
  double x;
  int i, k;
};
__device__ inline AppendFetch append_fetch(const View& v, int u, int j) {
  const int tid = threadIdx.x;
  const size_t cbase = (size_t)u * v.Mcap;
  AppendFetch f{0.0, 0, 0};
  if (tid < kHeadDim) f.x = (double)unit_R(v, u)[r_index(j, tid)];
  switch (tid - kHeadDim) {
    case 0: f.i = v.cn[cbase + j]; break;
    case 1: f.i = v.cb[cbase + j]; break;
    case 2: f.i = v.ctail[cbase + j]; break;
    case 3: f.i = v.cflag[cbase + j]; break;
    case 4: f.x = v.cM2[cbase + j]; break;
    case 5: f.x = v.tau[u]; break;
    case 6: f.i = v.nflag[u]; break;
    case 7: f.i = v.bump[u]; break;
    case 8: {
      f.i = v.free_top[u];
      f.k = f.i > 0 ? v.freelist[(size_t)u * v.Pcap + f.i - 1] : -1;
      break;
    }
    default: break;
  }
  return f;
}

// Cluster j (of M) receives token N of unit u.  Called by all NT >= 256 threads of the unit's workgroup with
// what append_fetch returned to each of them (the caller may have issued it long before).  The sum of UpdateVar
// is formed from 16 block sums computed side by side, and one thread then takes the decisions.
template <int NT>
__device__ inline void append_commit(const View& v, int u, int j, int M, int N, const void* kin, const void* vin,
                                     AppendSmem& a, const AppendFetch& f) {
  const int tid = threadIdx.x;
  const size_t cbase = (size_t)u * v.Mcap;
  const double r = f.x;
  switch (tid - kHeadDim) {
    case 0: a.cn = f.i; break;
    case 1: a.cb = f.i; break;
    case 2: a.ctail = f.i; break;
    case 3: a.cflag = f.i; break;
    case 4: a.m2 = f.x; break;
    case 5: a.tau = f.x; break;
    case 6: a.nflag = f.i; break;
    case 7: a.bump = f.i; break;
    case 8: a.free_top = f.i; a.free_page = f.k; break;
    default: break;
  }
  lds_barrier();
  // UpdateVar, element-wise part: delta_d = k_d - r_d, r'_d = r_d + delta_d / n'
  const int n1 = a.cn + 1;
  if (tid < kHeadDim) {
    const double dl = a.kd[tid] - r;
    a.delta[tid] = dl;
    a.r1[tid] = r + dl / (double)n1;
  }
  lds_barrier();
  if (tid < 16) {                           // block tid of sum_d delta_d * (k_d - r'_d)
    double s = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) s = fma(a.delta[tid * 8 + e], a.kd[tid * 8 + e] - a.r1[tid * 8 + e], s);
    a.bs[tid] = s;
  }
  lds_barrier();
  if (tid == 0) {
    const int sz = a.cn + a.cb;
    const int slot = sz % kPageTokens;
    int page = a.ctail;
    int ok = 1;
    a.nflag1 = a.nflag; a.top1 = a.free_top; a.bump1 = a.bump;
    if (slot == 0) {                      // no page yet, or the tail page is full
      int np = -1;                        // from the free stack, else from the untouched tail of the pool
      if (a.free_top > 0) {
        np = a.free_page;
        v.free_top[u] = a.free_top - 1;
        a.top1 = a.free_top - 1;
      } else if (a.bump < v.Pcap) {
        np = a.bump;
        v.bump[u] = a.bump + 1;
        a.bump1 = a.bump + 1;
      }
      if (np < 0) {
        v.err[u] |= DYNAKV_ERR_TOKENS;
        ok = 0;
      } else {
        v.pnext[(size_t)u * v.Pcap + np] = -1;
        if (sz != 0) v.pnext[(size_t)u * v.Pcap + page] = np;
        if (sz / kPageTokens < kInlinePages) v.cpg[(cbase + j) * kInlinePages + sz / kPageTokens] = np;
        v.ctail[cbase + j] = np;
        page = np;
      }
    }
    int commit = 0;
    if (ok) {
      v.last_assign[u] = j;
      if (a.cflag) {
        v.cb[cbase + j] = a.cb + 1;       // goes to the buffer of a flagged cluster
        v.csz[cbase + j] = a.cn + a.cb + 1;
      } else {
        // UpdateVar, the running part: M2' = M2 + sum_d delta_d * (k_d - r'_d)
        const double M2 = a.m2 + blocked16([&](int k) __attribute__((always_inline)) { return a.bs[k]; });
        const double var1 = M2 / (double)n1;
        bool trig = false;
        if (n1 >= 2 && !v.static_update) {
          if (v.var_alpha > 0.f && var1 > a.tau) trig = true;
          if (v.size_factor > 0.f && (double)n1 * (double)M > (double)v.size_factor * (double)(N + 1)) trig = true;
        }
        if (!trig) {
          v.cn[cbase + j] = n1;
          v.csz[cbase + j] = n1 + a.cb;
          v.cM2[cbase + j] = M2;
          commit = 1;
        } else {
          v.cflag[cbase + j] = 1;
          v.cb[cbase + j] = 1;
          v.csz[cbase + j] = a.cn + 1;
          v.flist[cbase + a.nflag] = j;
          v.nflag[u] = a.nflag + 1;
          a.nflag1 = a.nflag + 1;
        }
      }
      v.N[u] = N + 1;
      v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + slot] = N;
    }
    a.ok = ok; a.commit = commit; a.page = page; a.slot = slot;
  }
  lds_barrier();
  if (!a.ok) return;
  if (a.commit && tid < kHeadDim) store_centroid(v, u, j, tid, (float)a.r1[tid]);
  char* pg = page_ptr(v, u, a.page);
  if (tid < kHeadDim) copy_elem(pg, k_index(v.dtype, a.slot, tid), kin, (size_t)u * kHeadDim + tid, v.dtype);
  else if (tid < 2 * kHeadDim)
    copy_elem(pg, v_index(v.dtype, a.slot, tid - kHeadDim), vin, (size_t)u * kHeadDim + tid - kHeadDim, v.dtype);
}

// Workgroup-wide arg-min over (value, index) pairs, one per thread (index < 0: none); equal values go to the
// lowest index.  NT / 64 <= 16 wavefronts; sv / si need 16 entries.  Every thread gets the winning index.
template <int NT>
__device__ inline int block_argmin(double val, int idx, double* sv, int* si) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double ov = __shfl_xor(val, o);
    const int oi = __shfl_xor(idx, o);
    if (oi >= 0 && (idx < 0 || ov < val || (ov == val && oi < idx))) { val = ov; idx = oi; }
  }
  lds_barrier();
  if (lane == 0) { sv[w] = val; si[w] = idx; }
  lds_barrier();
  val = sv[0]; idx = si[0];
#pragma unroll
  for (int k = 1; k < NT / 64; ++k) {
    const double ov = sv[k];
    const int oi = si[k];
    if (oi >= 0 && (idx < 0 || ov < val || (ov == val && oi < idx))) { val = ov; idx = oi; }
  }
  return idx;
}

}  // namespace dynakv
