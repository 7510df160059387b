// Shared declarations of the gfx950 library: the device-side view of an index, the page layout,
// and small block-level helpers.  Everything here is for the HIP path only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dynakv.h"

namespace dynakv {

constexpr int kHeadDim = 128;
constexpr int kPageTokens = 16;                 // tokens per page = one MFMA tile of rows
constexpr int kPageElems = 2 * kPageTokens * kHeadDim;  // K region then V region
constexpr int kMaxClusters = 131072;            // per unit (the selection packs an id into 18 bits)
constexpr int kMaxInitClusters = 8192;          // clusters built at prefill
constexpr int kSelectLds = 16384;               // clusters whose scores and sizes the selection keeps in LDS; beyond,
                                                // it reads them from memory in every pass
constexpr int kMaxPrefill = 16384;              // k-means sorts one unit's labels in LDS
constexpr int kFusedClusters = 4096;            // clusters per unit the single-kernel retrieval can hold in LDS
constexpr int kMaxSplitMembers = 4096;          // largest cluster the split kernel handles
constexpr int kMaxKvSplits = 64;
constexpr int kCounters = 8;
constexpr int kLocalWindowMax = 128, kLocalClustersMax = 32;   // local update: largest window and cluster count
constexpr int kInlinePages = 8;                 // pages of a cluster found without walking its chain                // workgroups that share one unit's gathered pages

typedef float f4 __attribute__((ext_vector_type(4)));

// Device-side view of one index.  All arrays live in the caller's workspace.
struct View {
  // configuration
  int U, G, dtype, M0, Mcap, Ncap, Pcap, Lcap, Bmax, group_reduce, S, NW, fuse;
  int search_mean;   // the searches read the float32 means (always for float32 storage), else the 16-bit search copy
  int score_round;   // float64 scores are rounded to float32 before they are compared
  int static_update; // static-update baseline: nothing is ever flagged
  int token_level;   // every appended entry becomes a cluster of its own (baseline without clustering; local update)
  int local_W, local_k;  // local update: entries per local clustering and clusters it forms (0: not this mode)
  size_t Rstride;    // floats of centroid table per unit
  float var_alpha, size_factor, scale_f;
  double scale_d;
  // per unit
  int* M;            // [U] clusters in use
  int* N;            // [U] tokens stored
  int* err;          // [U] sticky DYNAKV_ERR_* bits
  double* tau;       // [U] split threshold on the variance
  int* nflag;        // [U] clusters currently flagged
  int* n_sel;        // [U] clusters selected by the last retrieval
  int* t_sel;        // [U] entries gathered by the last retrieval
  int* n_list;       // [U] entries in the gather list
  int* ticket;       // [U] arrival counter of the split-KV workgroups
  int NB;            // blocks of 256 clusters per unit (ceil(Mcap / 256))
  double* near_d;    // [U][NB] float32 means only: nearest cluster of the step's new key among clusters 256b .. 256b+255,
  int* near_j;       //         left by the score kernel of a whole decode step for the append that follows it
  float* near_zb;    // [U][4 NB] 16-bit search copy only: per wavefront of the score kernel (64 clusters), the largest z_j
  float* near_z2;    //           of the step's new key, the second largest, and the cluster of the largest (< 0: none)
  int* near_zj;
  float* zdist;      // [U][Mcap] 16-bit search copy only: z_j = <k_new, r~_j> - |r~_j|^2 / 2 of the step's new key as the
                     // matrix cores computed it (largest = nearest), for the append to pick from
  int* lcount;       // [U] local update: entries appended since the last local clustering
  int* rmax2;        // [U] bits of the largest |r~_j|^2 seen by a score pass since the index was built (a float >= 0)
  int* bump;         // [U] pages handed out from the pool so far
  int* free_top;     // [U] entries on the free-page stack
  int* last_assign;  // [U]
  long long* counters;  // [U][8] splits, failed, forced, (unused), entries gathered, retrievals, clusters scored, -
  // per cluster [U][Mcap]
  float* R;          // [U][Rstride] centroids, lane-interleaved: see r_index()
  uint16_t* Rq;      // [U][Rstride] the same centroids rounded to the 16-bit storage type (see rq_index()): the
                     // copy that the searches of a decode step read; unused for float32 storage
  int* cn;           // committed size n_j
  int* csz;          // stored entries n_j + |Buf_j| (kept beside the two so that the selection reads one array)
  int* cb;           // buffered entries |Buf_j|
  int* cflag;        // f_j
  int* flist;        // ids of the flagged clusters, first nflag[u] entries, in no particular order
  double* cM2;       // M2_j
  int* cpg;          // [.][8] first pages of the cluster (-1: none); later pages follow pnext
  int* ctail;        // last page
  float* score;      // last scores
  int* sel_ids;      // the active set in the order it is attended: ascending id, or (selection with its keys in memory) descending score
  unsigned char* in_req;  // membership in the last active set
  int* tok_off;      // scratch: exclusive prefix of sizes in score order
  int* pg_off;       // scratch: exclusive prefix of gather-list entry counts in score order
  // pages [U][Pcap]
  char* pages;       // [U][Pcap][kPageElems * elem size]
  int* ppos;         // [U][Pcap][16] token position of every slot
  int* pnext;        // [U][Pcap] next page of the same cluster (-1: last)
  int* freelist;     // [U][Pcap] stack of recycled pages
  // gather list [U][Lcap]: one entry per aligned group of four token slots of a page
  int* plist;        // page * 16 + group * 4 + (valid tokens - 1)
  int* plist_off;    // gather offset of the entry's first token
  // split-KV partial results
  float* part;       // [U][S][G][130]: 128 accumulators, running max (log2 domain), denominator
  // k-means / split scratch [U][Ncap]
  int* labels;
  int* order;        // positions sorted by (label, position)
  double* dist;
  int* koff;         // [U][Mcap+1] start of every cluster in `order`
  // k-means distance filter on the matrix cores
  uint16_t* kmA;     // [U][kmA_stride] centroids split into 16-bit terms, in A-operand order (see kmeans.hip)
  size_t kmA_stride; // 16-bit elements per unit
  float* hn;         // [U][Mpad32] -|r_j|^2 / 2 (-inf for padding rows)
  float* rmax;       // [U] max_j |r_j|
  int* nflagged;     // [U] points whose filter gap is below the rounding bound (listed in `order`)
  int* has_empty;    // [U] some cluster got no point in the last assignment
  int* xrange;       // [U][2] smallest and largest binary exponent among the unit's non-zero prefill keys
};

__host__ __device__ inline int elem_size(int dtype) { return dtype == DYNAKV_F32 ? 4 : 2; }

// ---- page layout -----------------------------------------------------------------------------
// A page stores 16 tokens: a K region and a V region, each [16 slots][128], one row per token, so that the
// bytes fetched follow the valid tokens exactly: a page with n valid tokens costs n K rows and n V rows.
// In the attention kernels lane l holds token slot l%16 and, per piece s, the 16 bytes at row offset
// 64*s + 16*(l/16) of that token's K row and of its V row (dims 32s + 8*(l/16) + e for 16-bit types, 16s +
// 4*(l/16) + i for float32): four lanes cover one 64-byte sector of one token.  QK^T consumes the K pieces as
// loaded; PV wants the four tokens of one column together, so the V pieces are transposed on chip.
// Every load of a slot is masked by the cluster's size, so slots that hold no token are never read and pages
// need no initialisation.
// Offsets are in elements from the start of the page; the V region starts at 2048.
__host__ __device__ inline int k_index16(int slot, int d) { return slot * kHeadDim + d; }
__host__ __device__ inline int v_index16(int slot, int d) { return 2048 + slot * kHeadDim + d; }
__host__ __device__ inline int k_index32(int slot, int d) { return slot * kHeadDim + d; }
__host__ __device__ inline int v_index32(int slot, int d) { return 2048 + slot * kHeadDim + d; }
__host__ __device__ inline int k_index(int dtype, int slot, int d) {
  return dtype == DYNAKV_F32 ? k_index32(slot, d) : k_index16(slot, d);
}
__host__ __device__ inline int v_index(int dtype, int slot, int d) {
  return dtype == DYNAKV_F32 ? v_index32(slot, d) : v_index16(slot, d);
}

// ---- centroid table ------------------------------------------------------------------------------
// Centroids are read by kernels in which lane l of a wavefront owns cluster 64*t + l.  The table is laid
// out so that such a wavefront reads 16 contiguous bytes per lane: [tile of 64 clusters][d/4][64][4].
__host__ __device__ inline size_t r_index(int j, int d) {
  return ((size_t)(j >> 6) * (kHeadDim / 4) + (d >> 2)) * 256 + (size_t)(j & 63) * 4 + (d & 3);
}
__host__ __device__ inline size_t r_stride(int Mcap) { return (size_t)((Mcap + 63) / 64) * 64 * kHeadDim; }
__device__ inline float* unit_R(const View& v, int u) { return v.R + (size_t)u * v.Rstride; }

// The representatives that a search reads (query similarity, Section 4.1; nearest cluster of a new entry,
// Algorithm 1) are kept in the storage type of the keys, like the entries they stand for (unless the configuration
// asks for the float32 means); the float32 table above stays the master copy for the statistics.  The 16-bit copy
// is stored as the B operand of v_mfma_f32_16x16x32_{f16,bf16}: [tile of 16 clusters][chunk of 32 coordinates]
// [lane][8], lane = 16 * (slice of 8 coordinates inside the chunk) + cluster inside the tile, so that lane l of a
// wavefront reads its 16 bytes of chunk c of tile T at byte offset ((4 T + c) * 64 + l) * 16: 1 KB contiguous per
// load, a whole tile (4 KB) per four loads.
__host__ __device__ inline size_t rq_index(int j, int d) {
  return ((((size_t)(j >> 4) * 4 + (d >> 5)) * 64 + ((d >> 3) & 3) * 16 + (j & 15)) << 3) + (d & 7);
}
constexpr int kTileClusters = 16;                       // clusters per tile of the search copy
constexpr int kTileElems = kTileClusters * kHeadDim;    // 16-bit elements per tile
__device__ inline uint16_t* unit_Rq(const View& v, int u) { return v.Rq + (size_t)u * v.Rstride; }
// float32 -> 16-bit storage type, round to nearest even; the bits.
__device__ inline uint16_t round_bits16(float x, int dtype) {
  if (dtype == DYNAKV_F16) return __builtin_bit_cast(uint16_t, (_Float16)x);
  const uint32_t u = __float_as_uint(x);
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);       // bfloat16 (centroids are finite)
}
// Writes coordinate d of centroid j: the float32 master and, for 16-bit storage, the search copy.
__device__ inline void store_centroid(const View& v, int u, int j, int d, float val) {
  unit_R(v, u)[r_index(j, d)] = val;
  if (v.dtype != DYNAKV_F32) unit_Rq(v, u)[rq_index(j, d)] = round_bits16(val, v.dtype);
}

// ---- the fixed summation order ----------------------------------------------------------------------
// Every float64 sum over the 128 coordinates runs in one order: blocks of 8 consecutive coordinates are
// accumulated left to right from zero (one fused multiply-add per term), and the 16 block sums are added left
// to right.  Dependency chains stay short, and the value is the same whether one lane owns the whole sum or 16
// lanes own one block each.

// One thread: block_sum(k) returns the sum of block k (k = 0..15, called in ascending k).
template <class F>
__device__ __forceinline__ double blocked16(F&& block_sum) {
  double total = 0.0;
#pragma unroll 4
  for (int k = 0; k < 16; ++k) total += block_sum(k);
  return total;
}
// Four consecutive lanes (one DPP quad), lane q holding the sums of blocks 4q..4q+3 in bs[]: every lane of
// the quad gets the total ((s0 + s1) + s2) + ... + s15, added strictly left to right.
__device__ inline double blocked16_quad(const double (&bs)[4]) {
  const int q = threadIdx.x & 3;
  double t = 0.0;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    double in = 0.0;
    if (r > 0) {   // running total of the lane to the left: quad_perm [0, 0, 1, 2]
      const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(t), 0x90, 0xF, 0xF, false);
      const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(t), 0x90, 0xF, 0xF, false);
      in = __hiloint2double(hi, lo);
    }
    const double mine = (((in + bs[0]) + bs[1]) + bs[2]) + bs[3];
    if (q == r) t = mine;
  }
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(t), 0xFF, 0xF, 0xF, false);   // quad_perm [3, 3, 3, 3]
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(t), 0xFF, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}

// Centroid j of the lane-interleaved table against NACC operands at once: out[a] = sum over d of the terms that
// term(d, r_d, acc) adds into acc[a] with one fma each, in the order above.  The loads of the next 32
// coordinates are in flight while the current 32 are consumed; `cur` holds coordinates 0..31, loaded by the
// caller with load_centroid_head (so that it can issue them before anything else it waits for).
__device__ inline void load_centroid_head(const float* R, int j, f4 (&first)[8]) {
  const f4* r = (const f4*)(R + r_index(j, 0));
#pragma unroll
  for (int i = 0; i < 8; ++i) first[i] = r[i * 64];
}
// Coordinates 32b .. 32b+31 (held in cur) of the sums: four blocks of 8.
template <int NACC, bool LEAN, class F>
__device__ __forceinline__ void centroid_batch(int b, const f4 (&cur)[8], double (&out)[NACC], F&& term) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    double acc[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a) acc[a] = 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int e = 0; e < 4; ++e) term(b * 32 + k * 8 + i * 4 + e, cur[k * 2 + i][e], acc);
      if (LEAN) asm volatile("" ::: "memory");   // lean variant: operand loads stay four coordinates deep
    }
#pragma unroll
    for (int a = 0; a < NACC; ++a) out[a] += acc[a];
    __builtin_amdgcn_sched_barrier(0);   // keeps the operand loads of later blocks from piling up in registers
  }
}
template <int NACC, bool PREFETCH = true, class F>
__device__ __forceinline__ void centroid_sums(const float* R, int j, f4 (&cur)[8], double (&out)[NACC], F&& term) {
  const f4* r = (const f4*)(R + r_index(j, 0));
#pragma unroll
  for (int a = 0; a < NACC; ++a) out[a] = 0.0;
#pragma unroll 1
  for (int b = 0; b < 3; ++b) {
    if constexpr (PREFETCH) {
      f4 nxt[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) nxt[i] = r[((b + 1) * 8 + i) * 64];
      centroid_batch<NACC, false>(b, cur, out, term);
#pragma unroll
      for (int i = 0; i < 8; ++i) cur[i] = nxt[i];
    } else {
      centroid_batch<NACC, true>(b, cur, out, term);
#pragma unroll
      for (int i = 0; i < 8; ++i) cur[i] = r[((b + 1) * 8 + i) * 64];
    }
  }
  centroid_batch<NACC, !PREFETCH>(3, cur, out, term);
  // the sums are complete here: without this, the compiler moves the last batch's arithmetic (not its operand
  // loads) into whatever conditional block first uses the result, and the loaded operands pile up in registers
#pragma unroll
  for (int a = 0; a < NACC; ++a) asm volatile("" : "+v"(out[a]));
}

// ---- element access -----------------------------------------------------------------------------
__device__ inline float bf16_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ inline float f16_to_float(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

// Element `i` of an array of the index's storage type, as float (exact).
__device__ inline float load_elem(const void* base, size_t i, int dtype) {
  if (dtype == DYNAKV_F32) return ((const float*)base)[i];
  const uint16_t h = ((const uint16_t*)base)[i];
  return dtype == DYNAKV_F16 ? f16_to_float(h) : bf16_to_float(h);
}
// Copies element `i` of `src` to element `j` of `dst` (same storage type, bits unchanged).
__device__ inline void copy_elem(void* dst, size_t j, const void* src, size_t i, int dtype) {
  if (dtype == DYNAKV_F32) ((uint32_t*)dst)[j] = ((const uint32_t*)src)[i];
  else ((uint16_t*)dst)[j] = ((const uint16_t*)src)[i];
}

// Eight consecutive elements starting at element i (i a multiple of 8), as floats: two 16-byte loads for
// float32, one for the 16-bit types.
__device__ inline void load8(const void* base, size_t i, int dtype, float (&x)[8]) {
  if (dtype == DYNAKV_F32) {
    const f4 a = *(const f4*)((const float*)base + i), b = *(const f4*)((const float*)base + i + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
  } else {
    const uint4 w = *(const uint4*)((const uint16_t*)base + i);
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint16_t h = (uint16_t)(ww[e >> 1] >> ((e & 1) * 16));
      x[e] = dtype == DYNAKV_F16 ? f16_to_float(h) : bf16_to_float(h);
    }
  }
}

__device__ inline char* page_ptr(const View& v, int u, int page) {
  return v.pages + ((size_t)u * v.Pcap + page) * ((size_t)kPageElems * elem_size(v.dtype));
}
// Key coordinate d of the token in `slot` of `page`, as float.
__device__ inline float page_key(const View& v, int u, int page, int slot, int d) {
  return load_elem(page_ptr(v, u, page), k_index(v.dtype, slot, d), v.dtype);
}

// ---- wavefront scans and reductions on DPP ----------------------------------------------------------
// Cross-lane moves inside a row of 16 lanes (row shifts, quad permutes, mirrors) and from one row to the next (row
// broadcasts) are operand modifiers of ordinary vector instructions: a 64-lane scan or reduction built from them
// costs a few dozen cycles, where the same built from lane permutes through LDS (what __shfl compiles to) costs a
// dependent LDS round trip per step.  A lane whose source lies outside its row, or whose row is masked out, gets 0.
template <int CTRL, int ROWS = 0xF>
__device__ __forceinline__ int dpp_or_zero(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, ROWS, 0xF, false); }
// A lane whose row is masked out keeps `old`.
template <int CTRL, int ROWS = 0xF>
__device__ __forceinline__ int dpp_or(int old, int x) { return __builtin_amdgcn_update_dpp(old, x, CTRL, ROWS, 0xF, false); }
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E;            // quad_perm [1,0,3,2], [2,3,0,1]
constexpr int kDppHalfMirror = 0x141, kDppMirror = 0x140;  // lane i <-> 7 - i inside 8 lanes, i <-> 15 - i inside a row
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;    // lane 15 of every row to the next row; lane 31 to rows 2 and 3
// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_incl_scan(int x) {
  x += dpp_or_zero<0x111>(x);            // row_shr:1, 2, 4, 8
  x += dpp_or_zero<0x112>(x);
  x += dpp_or_zero<0x114>(x);
  x += dpp_or_zero<0x118>(x);
  x += dpp_or_zero<kDppBcast15, 0xA>(x); // rows 1 and 3 add the total of the row before them
  x += dpp_or_zero<kDppBcast31, 0xC>(x); // rows 2 and 3 add the total of rows 0 and 1
  return x;
}
// Sum over the 64 lanes; every lane gets it.
__device__ __forceinline__ int wave_sum(int x) { return __builtin_amdgcn_readlane(wave_incl_scan(x), 63); }
// Largest value over the 64 lanes; every lane gets it.  (Butterfly inside each row, then row to row; a lane that a
// step does not reach keeps its own value, which leaves a maximum unchanged.)
__device__ __forceinline__ int wave_max(int x) {
  x = max(x, dpp_or<kDppXor1>(x, x));
  x = max(x, dpp_or<kDppXor2>(x, x));
  x = max(x, dpp_or<kDppHalfMirror>(x, x));
  x = max(x, dpp_or<kDppMirror>(x, x));
  x = max(x, dpp_or<kDppBcast15, 0xA>(x, x));
  x = max(x, dpp_or<kDppBcast31, 0xC>(x, x));
  return __builtin_amdgcn_readlane(x, 63);
}
__device__ __forceinline__ int wave_min(int x) { return -wave_max(-x); }

// ---- block helpers ------------------------------------------------------------------------------
// Workgroup barrier for data that travels through LDS only: it waits for this wavefront's LDS (and scalar)
// operations, not for its outstanding global loads and stores as __syncthreads() does.  A stage that has issued
// global stores (scores, active-set flags, list entries) or loads it will only need later then does not pay a
// memory round trip at every barrier.  Data that other threads of the workgroup read back from global memory
// still needs __syncthreads().
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
template <bool LDS_ONLY>
__device__ __forceinline__ void block_barrier() {
  if constexpr (LDS_ONLY) lds_barrier();
  else __syncthreads();
}

// Exclusive prefix sum over the threads of a block (blockDim.x a multiple of 64, at most 1024), or over its
// first 64 * nw threads if nw > 0 (then only those may call).
// `sm` needs 64 ints.  Returns the prefix of this thread; `total` receives the block sum.
template <bool LDS_ONLY = false>
__device__ inline int block_excl_scan(int val, int* sm, int& total, int nw = 0) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (nw == 0) nw = blockDim.x >> 6;
  const int x = wave_incl_scan(val);
  block_barrier<LDS_ONLY>();
  if (lane == 63) sm[w] = x;
  block_barrier<LDS_ONLY>();
  int base = 0, all = 0;
  for (int k = 0; k < nw; ++k) {
    const int t = sm[k];
    if (k < w) base += t;
    all += t;
  }
  total = all;
  return base + x - val;
}

// The same over 64-bit values (two 32-bit sums side by side); `sm` needs 16 entries.
template <bool LDS_ONLY = false>
__device__ inline unsigned long long block_excl_scan64(unsigned long long val, unsigned long long* sm,
                                                       unsigned long long& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  // the two halves are sums of their own (neither overflows 32 bits): two 32-bit scans
  const unsigned lo = (unsigned)wave_incl_scan((int)(unsigned)val), hi = (unsigned)wave_incl_scan((int)(unsigned)(val >> 32));
  const unsigned long long x = (unsigned long long)lo | ((unsigned long long)hi << 32);
  block_barrier<LDS_ONLY>();
  if (lane == 63) sm[w] = x;
  block_barrier<LDS_ONLY>();
  unsigned long long base = 0, all = 0;
  for (int k = 0; k < nw; ++k) {
    const unsigned long long t = sm[k];
    if (k < w) base += t;
    all += t;
  }
  total = all;
  return base + x - val;
}

// k-th page of the cluster with flat index cj (= u * Mcap + j); `prev` is its page k-1.
// Adds n to counter k of unit u without waiting for the old value (the counters are statistics: nothing in a
// kernel reads them back).
__device__ __forceinline__ void count(const View& v, int u, int k, long long n) {
  __hip_atomic_fetch_add(&v.counters[(size_t)u * kCounters + k], n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline int cluster_page(const View& v, int u, size_t cj, int k, int prev) {
  return k < kInlinePages ? v.cpg[cj * kInlinePages + k] : v.pnext[(size_t)u * v.Pcap + prev];
}

// Block-wide arg-min / arg-max over (value, index) pairs held one per thread of a 256-thread block; ties go
// to the lowest index; index < 0 means "no candidate".  Result in sv[0], si[0].
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

__device__ inline int pages_available(const View& v, int u) { return v.free_top[u] + (v.Pcap - v.bump[u]); }
__device__ inline void free_page(const View& v, int u, int page) {
  const int top = v.free_top[u];
  v.freelist[(size_t)u * v.Pcap + top] = page;
  v.free_top[u] = top + 1;
}

// ---- launchers (one per source file) ------------------------------------------------------------
hipError_t launch_build_index(const View& v, const void* K, const void* V, int n_tokens, const int* init_idx,
                              int iters, void* workspace, size_t workspace_bytes, hipStream_t st);
// kin != null: the scores' pass over the centroid table also leaves, per block of 256 clusters, the cluster nearest
// to the new key `kin` (near_d / near_j), for launch_append(.., prescanned = true).
hipError_t launch_score_select(const View& v, const void* Q, int budget, const void* kin, hipStream_t st);
hipError_t launch_near(const View& v, const void* kin, hipStream_t st);
bool retrieve_is_fused(const View& v);
hipError_t launch_retrieve_fused(const View& v, const void* Q, int budget, float* out, float* lse, const void* kin,
                                 const void* vin, bool split, hipStream_t st);
hipError_t launch_gather_attend(const View& v, const void* Q, float* out, float* lse, hipStream_t st);
// split: the unit's due splits follow in the same launch.
hipError_t launch_append(const View& v, const void* k, const void* val, bool prescanned, bool split, hipStream_t st);
hipError_t launch_split(const View& v, hipStream_t st);
hipError_t launch_local_recluster(const View& v, int iters, hipStream_t st);
hipError_t launch_extend(const View& v, const void* K, const void* V, int n, hipStream_t st);
hipError_t launch_export(const View& v, const dynakv_state_t& dst, hipStream_t st);
hipError_t launch_import(const View& v, const dynakv_state_t& src, hipStream_t st);
hipError_t launch_place(const View& v, const void* K, const void* V, int n_tokens, const void* Qref, int n_ref, int budget,
                        float* P, int* order, hipStream_t st);

}  // namespace dynakv
