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

// ---- the same by one wavefront ------------------------------------------------------------------------
// Lane l fetches coordinates l and l + 64 of the centroid, lanes 0..8 one field each of the cluster's record or of
// the unit's allocator state (the fields of AppendFetch, in the same order).
struct AppendFetchWave {
  double x0, x1, xf;
  int i, k;
};
__device__ inline AppendFetchWave append_fetch_wave(const View& v, int u, int j) {
  const int lane = threadIdx.x & 63;
  const size_t cbase = (size_t)u * v.Mcap;
  AppendFetchWave f{0.0, 0.0, 0.0, 0, 0};
  f.x0 = (double)unit_R(v, u)[r_index(j, lane)];
  f.x1 = (double)unit_R(v, u)[r_index(j, lane + 64)];
  switch (lane) {
    case 0: f.i = v.cn[cbase + j]; break;
    case 1: f.i = v.cb[cbase + j]; break;
    case 2: f.i = v.ctail[cbase + j]; break;
    case 3: f.i = v.cflag[cbase + j]; break;
    case 4: f.xf = v.cM2[cbase + j]; break;
    case 5: f.xf = v.tau[u]; break;
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
__device__ __forceinline__ double readlane_f64(double x, int lane) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), lane), __builtin_amdgcn_readlane(__double2loint(x), lane));
}
// Sum of a float64 over the 64 lanes (DPP butterfly inside the rows, row broadcasts across them); every lane gets it.
template <int CTRL, int ROWS>
__device__ __forceinline__ double dpp_f64(double x) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, ROWS, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, ROWS, 0xF, false);
  return __hiloint2double(hi, lo);           // a lane that the step does not reach gets +0.0
}
__device__ __forceinline__ double wave_sum_f64(double x) {
  x += dpp_f64<kDppXor1, 0xF>(x);
  x += dpp_f64<kDppXor2, 0xF>(x);
  x += dpp_f64<kDppHalfMirror, 0xF>(x);
  x += dpp_f64<kDppMirror, 0xF>(x);
  x += dpp_f64<kDppBcast15, 0xA>(x);
  x += dpp_f64<kDppBcast31, 0xC>(x);
  return readlane_f64(x, 63);
}
// append_commit by ONE wavefront, with no workgroup barrier: the other wavefronts of the workgroup are free to do
// something else meanwhile.  a.kd holds the new key; on return the fields of `a` that the plan of the splits reads
// (ok, cn, cb, slot, page, nflag1, top1, bump1) are in place, and every global store of the append has completed.
__device__ inline void append_commit_wave(const View& v, int u, int j, int M, int N, const void* kin, const void* vin,
                                          AppendSmem& a, const AppendFetchWave& f) {
  const int lane = threadIdx.x & 63;
  const size_t cbase = (size_t)u * v.Mcap;
  const int cn = __builtin_amdgcn_readlane(f.i, 0), cb = __builtin_amdgcn_readlane(f.i, 1);
  const int ctail = __builtin_amdgcn_readlane(f.i, 2), cflag = __builtin_amdgcn_readlane(f.i, 3);
  const double m2 = readlane_f64(f.xf, 4), tau = readlane_f64(f.xf, 5);
  const int nflag = __builtin_amdgcn_readlane(f.i, 6), bump = __builtin_amdgcn_readlane(f.i, 7);
  const int free_top = __builtin_amdgcn_readlane(f.i, 8), free_page = __builtin_amdgcn_readlane(f.k, 8);
  // UpdateVar: delta_d = k_d - r_d, r'_d = r_d + delta_d / n', M2' = M2 + sum_d delta_d (k_d - r'_d)
  const int n1 = cn + 1;
  const double k0 = a.kd[lane], k1 = a.kd[lane + 64];
  const double d0 = k0 - f.x0, d1 = k1 - f.x1;
  const double r0 = f.x0 + d0 / (double)n1, r1 = f.x1 + d1 / (double)n1;
  const double M2 = m2 + wave_sum_f64(fma(d0, k0 - r0, d1 * (k1 - r1)));
  // the decisions, by every lane alike (all operands are wavefront-uniform); lane 0 writes
  const int sz = cn + cb, slot = sz % kPageTokens;
  int page = ctail, ok = 1, nflag1 = nflag, top1 = free_top, bump1 = bump;
  if (slot == 0) {                        // no page yet, or the tail page is full
    int np = -1;                          // from the free stack, else from the untouched tail of the pool
    if (free_top > 0) { np = free_page; top1 = free_top - 1; }
    else if (bump < v.Pcap) { np = bump; bump1 = bump + 1; }
    if (np < 0) ok = 0;
    else {
      if (lane == 0) {
        v.free_top[u] = top1; v.bump[u] = bump1;
        v.pnext[(size_t)u * v.Pcap + np] = -1;
        if (sz != 0) v.pnext[(size_t)u * v.Pcap + page] = np;
        if (sz / kPageTokens < kInlinePages) v.cpg[(cbase + j) * kInlinePages + sz / kPageTokens] = np;
        v.ctail[cbase + j] = np;
      }
      page = np;
    }
  }
  int commit = 0;
  if (ok) {
    bool trig = false;
    if (!cflag && n1 >= 2 && !v.static_update) {
      if (v.var_alpha > 0.f && M2 / (double)n1 > tau) trig = true;
      if (v.size_factor > 0.f && (double)n1 * (double)M > (double)v.size_factor * (double)(N + 1)) trig = true;
    }
    commit = !cflag && !trig;
    if (!cflag && trig) nflag1 = nflag + 1;
    if (lane == 0) {
      v.last_assign[u] = j;
      if (cflag) {                          // goes to the buffer of a flagged cluster
        v.cb[cbase + j] = cb + 1;
        v.csz[cbase + j] = cn + cb + 1;
      } else if (!trig) {
        v.cn[cbase + j] = n1;
        v.csz[cbase + j] = n1 + cb;
        v.cM2[cbase + j] = M2;
      } else {
        v.cflag[cbase + j] = 1;
        v.cb[cbase + j] = 1;
        v.csz[cbase + j] = cn + 1;
        v.flist[cbase + nflag] = j;
        v.nflag[u] = nflag + 1;
      }
      v.N[u] = N + 1;
      v.ppos[((size_t)u * v.Pcap + page) * kPageTokens + slot] = N;
    }
    if (commit) { store_centroid(v, u, j, lane, (float)r0); store_centroid(v, u, j, lane + 64, (float)r1); }
    char* pg = page_ptr(v, u, page);
    copy_elem(pg, k_index(v.dtype, slot, lane), kin, (size_t)u * kHeadDim + lane, v.dtype);
    copy_elem(pg, k_index(v.dtype, slot, lane + 64), kin, (size_t)u * kHeadDim + lane + 64, v.dtype);
    copy_elem(pg, v_index(v.dtype, slot, lane), vin, (size_t)u * kHeadDim + lane, v.dtype);
    copy_elem(pg, v_index(v.dtype, slot, lane + 64), vin, (size_t)u * kHeadDim + lane + 64, v.dtype);
  } else if (lane == 0) {
    v.err[u] |= DYNAKV_ERR_TOKENS;
  }
  if (lane == 0) {
    a.cn = cn; a.cb = cb; a.ok = ok; a.commit = commit; a.page = page; a.slot = slot;
    a.nflag1 = nflag1; a.top1 = top1; a.bump1 = bump1;
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
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
