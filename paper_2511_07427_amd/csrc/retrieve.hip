// Decode, first half of a step (Algorithm 1, decode block: the top clusters by query-centroid similarity are
// loaded; Section 4.1; attention over the reordered entries, Section 7):
//   score kernels  - inner products <q_g, r_j> reduced over the query group: on the matrix cores over the 16-bit
//                    search copy (score.hpp), or in float64 over the float32 means
//   select_kernel  - order by (score desc, id asc), longest prefix under the token budget, gather list
//   gather_attend  - streams the selected clusters' pages once; QK^T and PV on matrix cores with an
//                    online (running-max) softmax, so any gather order is overflow-safe; split over
//                    several workgroups per unit and merged by the last one to arrive.
//   retrieve_fused - all of the above for one unit in one workgroup and, in a whole decode step, the append
//                    (Section 4.2) and the due splits as well: the step is one launch.
#include <type_traits>

#include "split.hpp"
#include "score.hpp"

namespace dynakv {

namespace {

// ------------------------------------------------------------------------------------------- scores
// (a) float32 means (float32 storage, or a configuration that asks for them): float64 on the vector units.
// Lane = cluster: the float32 table is lane-interleaved, so every load below is 1 KB contiguous per wavefront.
// NEAR: the same pass also finds, per workgroup (256 clusters), the cluster nearest to the step's new key (one
// more accumulator per centroid) and leaves it in near_d / near_j.
template <int GP, bool NEAR>
__global__ __launch_bounds__(256) void score_mean_kernel(View v, const void* Q, const void* kin) {
  constexpr int NA = GP + (NEAR ? 1 : 0);
  __shared__ double qs[kHeadDim][GP];
  __shared__ double kd[NEAR ? kHeadDim : 1];
  __shared__ double am_v[16];
  __shared__ int am_i[16];
  const int u = blockIdx.y, tid = threadIdx.x;
  const int j = blockIdx.x * 256 + tid;
  const float* R = unit_R(v, u);
  const int M = v.M[u];
  if (blockIdx.x * 256 >= M) return;
  f4 row[8];
  const bool live = (j & ~63) < M;                  // false: whole wavefront past the last cluster
  if (live) load_centroid_head(R, j, row);
  for (int t = tid; t < GP * kHeadDim; t += 256) {
    const int g = t / kHeadDim, d = t % kHeadDim;
    qs[d][g] = g < v.G ? (double)load_elem(Q, ((size_t)u * v.G + g) * kHeadDim + d, v.dtype) : 0.0;
  }
  if constexpr (NEAR)
    if (tid < kHeadDim) kd[tid] = (double)load_elem(kin, (size_t)u * kHeadDim + tid, v.dtype);
  __syncthreads();
  if (!NEAR && !live) return;
  double acc[NA];
  if (live) {
    centroid_sums<NA>(R, j, row, acc, [&](int d, float rv, double (&a)[NA]) __attribute__((always_inline)) {
      const double rd = (double)rv;
#pragma unroll
      for (int g = 0; g < GP; ++g) a[g] = fma(qs[d][g], rd, a[g]);
      if constexpr (NEAR) {
        const double t = kd[d] - rd;
        a[GP] = fma(t, t, a[GP]);
      }
    });
  }
  const bool mine = live && j < M;
  if (mine) {
    double red = acc[0];
#pragma unroll
    for (int g = 1; g < GP; ++g)
      if (g < v.G) red = v.group_reduce == DYNAKV_GROUP_MAX ? fmax(red, acc[g]) : red + acc[g];
    v.score[(size_t)u * v.Mcap + j] = (float)(red * v.scale_d);
  }
  if constexpr (NEAR) {
    const double dist = mine ? acc[NA - 1] : 0.0;
    const int jw = block_argmin<256>(dist, mine ? j : -1, am_v, am_i);
    if (mine && j == jw) {
      v.near_d[(size_t)u * v.NB + blockIdx.x] = dist;
      v.near_j[(size_t)u * v.NB + blockIdx.x] = j;
    }
  }
}

// (b) 16-bit search copy: matrix cores.  grid (workgroups per unit, U), four wavefronts, each taking groups of four
// tiles of 16 clusters: 16 KB per wavefront in flight, twice that while the next group is requested.  SCORES: rows 0..G-1 are the query heads and the scaled, group-reduced
// scores go to v.score; NEAR: row G is the step's new key and z_j = <k, r~_j> - |r~_j|^2 / 2 goes to v.zdist for
// the append kernel to pick the nearest cluster from.  The largest |r~_j|^2 is folded into v.rmax2.
template <bool BF, int NBLK, bool SCORES, bool NEAR>
__global__ __launch_bounds__(256) void score_mfma_kernel(View v, const void* Q, const void* kin) {
  const int u = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint4* tiles = (const uint4*)unit_Rq(v, u);
  // groups of 64 clusters (four tiles) are dealt round-robin to the wavefronts of the unit's workgroups
  const int g0 = blockIdx.x * 4 + wave, gstep = gridDim.x * 4;
  uint4 b[4][4], nb[4][4];
  auto fetch = [&](uint4 (&dst)[4][4], int g) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int s = 0; s < 4; ++s)
        dst[t][s] = (size_t)(g * 4 + t + 1) * kTileElems <= v.Rstride ? tiles[((size_t)(g * 4 + t) * 4 + s) * 64 + lane] : uint4{0, 0, 0, 0};
  };
  // the first M0 clusters exist in every state (M never drops below M0): their rows are requested before M is known
  const bool early = (g0 + 1) * 64 <= v.M0;
  if (early) fetch(b, g0);
  const int M = v.M[u];
  if (g0 * 64 >= M) return;
  if (!early) fetch(b, g0);
  ScoreRows<NBLK> A;
  load_score_rows<NBLK>(A, SCORES ? v.G : 0, Q, NEAR ? kin : nullptr, u, lane);
  const int G = SCORES ? v.G : 0;
  float rmax2 = 0.f;
  for (int g = g0; g * 64 < M; g += gstep) {
    const bool more = (g + gstep) * 64 < M;
    if (more) fetch(nb, g + gstep);                   // the next group's rows are in flight while this one is consumed
    float zb = -__builtin_inff(), z2 = -__builtin_inff();
    int jb = -1;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if ((g * 4 + t) * kTileClusters >= M) break;
      float red, kdot, nrm2;
      score_tile<BF, NBLK, NEAR>(b[t], A, G, v.group_reduce, lane, red, kdot, nrm2);
      const int j = (g * 4 + t) * kTileClusters + lane;
      if (lane < kTileClusters && j < M) {
        if constexpr (SCORES) v.score[(size_t)u * v.Mcap + j] = red * v.scale_f;
        if constexpr (NEAR) {
          const float z = kdot - 0.5f * nrm2;
          v.zdist[(size_t)u * v.Mcap + j] = z;
          if (jb < 0 || z > zb) { z2 = jb < 0 ? z2 : zb; zb = z; jb = j; }
          else z2 = fmaxf(z2, z);
        }
        rmax2 = fmaxf(rmax2, nrm2);
      }
    }
    if constexpr (NEAR) {             // this group's 64 clusters: best, its cluster, runner-up
      wave_best2(zb, jb, z2);
      if (lane == 0) {
        const size_t w = (size_t)u * v.NB * 4 + g;
        v.near_zb[w] = zb; v.near_z2[w] = z2; v.near_zj[w] = jb;
      }
    }
    if (more) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int s = 0; s < 4; ++s) b[t][s] = nb[t][s];
    }
  }
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) rmax2 = fmaxf(rmax2, __shfl_xor(rmax2, o));
  if (lane == 0) atomicMax(&v.rmax2[u], __float_as_int(rmax2));      // non-negative floats order like their bits
}

// ------------------------------------------------------------------------------------------- selection
__device__ inline uint32_t orderable(float f) {
  const uint32_t b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int kIdBits = 18, kIdMask = (1 << kIdBits) - 1;   // a candidate's key: score above, kIdMask - id below
static_assert(kMaxClusters <= kIdMask + 1, "cluster ids must fit the candidate keys");
constexpr int kCountMax = 1024;     // selected clusters ordered by counting; larger selections take the full sort
constexpr int kSelRegion = kCountMax * 12;   // bytes of candidate keys (8) and sizes (4)

// LDS of the selection.  `region` holds the candidates of the fast path (or the ids of the full sort) and
// needs max(kSelRegion, 2 * Mpad) bytes; `list` receives the first `list_cap` gather-list entries.
// What the selection needs to retake the budget cut in float64 (16-bit search copy only): eps = bound on the error
// of a float32 score (0: scores are exact, nothing is retaken), Q = the queries.
struct SelectExact {
  float eps;
  const void* Q;
};
constexpr int kBandMax = 64;        // clusters within the bound of the cut that are re-scored in float64

__device__ inline float unorderable(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

struct SelectLds {
  uint32_t* skey;          // [Mpad] orderable scores, padded with 0 up to the next power of two; null: the scores are
                           // read from the workspace in every pass (more clusters than LDS holds)
  const int* sw;           // [M] stored sizes, or null: they are read from the workspace
  unsigned char* region;
  int* hist;               // [4][256]
  int* srt;                // [CMAX] sizes in rank order; may alias sw, must not alias hist or list
  int* sm;                 // [64]
  int* misc;               // [8]
  int* list;
  int list_cap;
  unsigned* selbits;       // [ceil(M / 32)] zeroed by the caller, or null: bit j is set for every selected cluster j, so that
                           // threads of the same workgroup can read the active set without a trip through memory
};

// List entries of one page holding nv tokens, from list position w and gather offset t0 on.
__device__ __forceinline__ void emit_page(int page, int nv, int w, int t0, int* plist, int* poff, int* lds_list,
                                          int lds_cap) {
  for (int qd = 0; 4 * qd < nv; ++qd) {
    const int e = page * 16 + qd * 4 + (min(4, nv - 4 * qd) - 1);
    plist[w + qd] = e;
    if (w + qd < lds_cap) lds_list[w + qd] = e;
    poff[w + qd] = t0 + 4 * qd;
  }
}

// Gather-list entry: one aligned group of four token slots ("quad") of a page,
// page * 16 + quad * 4 + (valid tokens - 1); its gather offset is that of its first token.

// Selection for one unit, run by a whole workgroup of NT threads (NT >= 256).  Clusters are ordered by
// (score desc, id asc); the active set is the longest prefix of that order whose stored sizes fit the budget
// (or the best cluster alone, cut to the budget, if even that one does not fit).  Records the active set and
// writes the gather list: in ascending cluster id where keys, sizes and the set's bitmap are in LDS (emit_by_id;
// no selected cluster is ranked), in score order otherwise.  Returns the number of gather-list entries.
//
// Puts the positions 0 .. cut-1 of the candidate keys ck into 256 bins by the leading bits in which the keys'
// scores differ (counting sort, bins in descending order) and returns the shift that yields a key's bin:
// ((key >> 16) >> shift) & 255.  hist[0..255]: bin sizes, [256..511]: candidates in higher bins, [512..767]: fill
// counters; misc[0..1]: scratch; lst: the positions in bin order.  Whole workgroup; kept out of line, it is rarely
// needed.
template <int NT>
__device__ __noinline__ int bin_candidates(int* hist, int* misc, int* lst, const unsigned long long* ck, int cut) {
  const int tid = threadIdx.x, lane = tid & 63;
  if (tid == 0) { misc[0] = -1; misc[1] = 0; }
  for (int i = tid; i < 768; i += NT) hist[i] = 0;
  lds_barrier();
  uint32_t lo = 0xFFFFFFFFu, hi = 0u;
  for (int p = tid; p < cut; p += NT) {
    const uint32_t k = (uint32_t)(ck[p] >> kIdBits);
    lo = min(lo, k); hi = max(hi, k);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { lo = min(lo, (uint32_t)__shfl_xor((int)lo, o)); hi = max(hi, (uint32_t)__shfl_xor((int)hi, o)); }
  if (lane == 0) { atomicMin((unsigned*)&misc[0], lo); atomicMax((unsigned*)&misc[1], hi); }
  lds_barrier();
  const uint32_t differ = (uint32_t)misc[0] ^ (uint32_t)misc[1];
  const int shift = differ ? max(31 - __clz((int)differ) - 7, 0) : 0;
  for (int p = tid; p < cut; p += NT) atomicAdd(&hist[((uint32_t)(ck[p] >> kIdBits) >> shift) & 255u], 1);
  lds_barrier();
  if (tid < 64) {                      // lane l owns the bins 255 - 4l .. 252 - 4l, highest first
    int hv[4], t = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) { hv[k] = hist[255 - (4 * lane + k)]; t += hv[k]; }
    int inc = t;
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(inc, o);
      if (lane >= o) inc += y;
    }
    int run = inc - t;
#pragma unroll
    for (int k = 0; k < 4; ++k) { hist[256 + 255 - (4 * lane + k)] = run; run += hv[k]; }
  }
  lds_barrier();
  for (int p = tid; p < cut; p += NT) {
    const int d = ((uint32_t)(ck[p] >> kIdBits) >> shift) & 255u;
    lst[hist[256 + d] + atomicAdd(&hist[512 + d], 1)] = p;
  }
  lds_barrier();
  return shift;
}

// Calls f(j, key of cluster j) for the clusters j = tid, tid + NT, ... < M of the calling thread; four keys are
// requested at a time, so that passes which read them from memory pay the latency once per four.
template <int NT, class KeyAt, class F>
__device__ __forceinline__ void for_each_key(int M, KeyAt&& key_at, F&& f) {
  for (int j0 = threadIdx.x; j0 < M; j0 += 4 * NT) {
    uint32_t kk[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) kk[i] = j0 + i * NT < M ? key_at(j0 + i * NT) : 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (j0 + i * NT < M) f(j0 + i * NT, kk[i]);
  }
}

// Exclusive prefix sums of three ints over the threads of a block at once (blockDim.x a multiple of 64, at most
// 1024); `sm` needs 48 ints.  a, b, c become the prefixes, ta, tb, tc the block sums.
template <bool LDS_ONLY>
__device__ inline void block_excl_scan3(int& a, int& b, int& c, int* sm, int& ta, int& tb, int& tc) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int xa = wave_incl_scan(a), xb = wave_incl_scan(b), xc = wave_incl_scan(c);
  block_barrier<LDS_ONLY>();
  if (lane == 63) { sm[3 * w] = xa; sm[3 * w + 1] = xb; sm[3 * w + 2] = xc; }
  block_barrier<LDS_ONLY>();
  int ba = 0, bb = 0, bc = 0;
  ta = 0; tb = 0; tc = 0;
  for (int k = 0; k < nw; ++k) {
    const int ya = sm[3 * k], yb = sm[3 * k + 1], yc = sm[3 * k + 2];
    if (k < w) { ba += ya; bb += yb; bc += yc; }
    ta += ya; tb += yb; tc += yc;
  }
  a = ba + xa - a; b = bb + xb - b; c = bc + xc - c;
}

// Records the active set held in s.selbits and writes its gather list, in ascending cluster id: thread t takes the
// R = ceil(M / NT) <= MAXR (8 or 16) clusters t R .. t R + R - 1 (sizes in s.sw), one block-wide prefix sum places
// every cluster's entries.  No cluster is ranked: the order in which selected clusters are attended does not matter
// to the method.  Page tables are requested and lists written eight clusters at a time.
// take_all >= 0: the one selected cluster contributes this many entries instead of its size.
// Returns the number of gather-list entries; the caller's barrier makes the list in LDS visible.
template <int NT, int MAXR>
__device__ inline int emit_by_id(const View& v, int u, int M, const SelectLds& s, int take_all) {
  static_assert(MAXR == 8 || MAXR == 16, "rounds of eight clusters");
  const int tid = threadIdx.x;
  const size_t cb = (size_t)u * v.Mcap;
  const int R = max(1, (M + NT - 1) / NT);               // workgroup-uniform
  const int j0 = tid * R;
  unsigned bits = 0;
  if (j0 < M) {                                          // the R bits from j0 on (they may straddle two words)
    const int wd = j0 >> 5, sh = j0 & 31;
    const unsigned lo = s.selbits[wd], hi = sh + R > 32 ? s.selbits[wd + 1] : 0u;
    bits = (unsigned)((((unsigned long long)hi << 32) | lo) >> sh) & ((1u << R) - 1u);
  }
  int w[MAXR];
  int tok = 0, quads = 0, cnt = 0;
  int4 pa[8], pb[8];
  // the page tables of a round's clusters are requested together and used once their places in the list are known
  auto request = [&](int base) __attribute__((always_inline)) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pa[e] = int4{-1, -1, -1, -1}; pb[e] = int4{-1, -1, -1, -1};
      if (base + e < R && ((bits >> (base + e)) & 1u)) {
        const int4* row = (const int4*)&v.cpg[(cb + j0 + base + e) * kInlinePages];
        pa[e] = row[0];
        if (w[base + e] > 4 * kPageTokens) pb[e] = row[1];
      }
    }
  };
#pragma unroll
  for (int e = 0; e < MAXR; ++e) {
    w[e] = 0;
    if (e < R && ((bits >> e) & 1u)) {
      w[e] = take_all >= 0 ? take_all : s.sw[j0 + e];
      tok += w[e]; quads += (w[e] + 3) >> 2; ++cnt;
    }
  }
  request(0);
  int t_tok, t_quads, t_cnt;
  block_excl_scan3<true>(tok, quads, cnt, s.sm, t_tok, t_quads, t_cnt);
  int* plist = v.plist + (size_t)u * v.Lcap;
  int* poff = v.plist_off + (size_t)u * v.Lcap;
#pragma unroll
  for (int base = 0; base < MAXR; base += 8) {
    if (base >= R) break;                                // workgroup-uniform
    if (base > 0) request(base);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (base + e >= R) break;                          // workgroup-uniform
      if (!((bits >> (base + e)) & 1u)) continue;
      v.sel_ids[cb + cnt] = j0 + base + e;
      const int take = w[base + e], npages = (take + kPageTokens - 1) / kPageTokens;
      const int pgs[kInlinePages] = {pa[e].x, pa[e].y, pa[e].z, pa[e].w, pb[e].x, pb[e].y, pb[e].z, pb[e].w};
      int page = -1;
#pragma unroll
      for (int k = 0; k < kInlinePages; ++k)
        if (k < npages) {
          page = pgs[k];
          if (page >= 0)
            emit_page(page, min(kPageTokens, take - k * kPageTokens), quads + 4 * k, tok + k * kPageTokens, plist, poff,
                      s.list, s.list_cap);
        }
      for (int kk = kInlinePages; kk < npages && page >= 0; ++kk) {    // pages past the inline table: walk the chain
        page = v.pnext[(size_t)u * v.Pcap + page];
        if (page >= 0)
          emit_page(page, min(kPageTokens, take - kk * kPageTokens), quads + 4 * kk, tok + kk * kPageTokens, plist, poff,
                    s.list, s.list_cap);
      }
      tok += take; quads += (take + 3) >> 2; ++cnt;
    }
  }
  if (tid == 0) {
    v.n_sel[u] = t_cnt; v.t_sel[u] = t_tok; v.n_list[u] = t_quads; v.ticket[u] = 0;
    count(v, u, 4, t_tok);
    count(v, u, 5, 1);
    count(v, u, 6, M);
  }
  return t_quads;
}

// No cluster outside the active set is ever ordered.  The score at which the running size first exceeds the budget
// is found by a radix search over the 32-bit orderable scores (four passes of size-weighted 256-bin histograms);
// everything above it is selected, equal scores are taken by ascending id while they fit.  With keys, sizes and
// the active set's bitmap in LDS (s.skey, s.sw, s.selbits; at most MAXR clusters per thread) the gather list then
// follows the cluster ids (emit_by_id).  Otherwise (more clusters than LDS holds) each selected cluster finds its
// rank and its gather offsets by counting the selected clusters that precede it: the list is in score order, and at
// most CMAX clusters can be selected (more: the retrieval is cut short and DYNAKV_ERR_SELECT is set).
// first_ready: the caller has zeroed s.hist and set s.misc (entry 4 = 0x7fffffff, the others 0), has added every
// cluster's size to bin (key >> 24) of the first histogram, and a barrier lies behind all of that.
//
// Scores computed in float32 on the matrix cores carry an error of at most ex.eps.  The cut that exact scores
// would give lies within eps of the float32 one, so every cluster more than 2 eps above it is selected and every
// cluster more than 2 eps below it is not, whatever the exact values; the clusters in between (the band, normally
// the cluster at the cut alone) are re-scored in float64 by the first wavefront and taken in exact order while
// they fit.  The selected SET is therefore that of exact arithmetic.  Bands of more than kBandMax clusters
// (degenerate inputs: many equal scores) are resolved on the float32 scores alone.
template <int NT, int CMAX = kCountMax, int MAXR = 8>
__device__ inline int select_phase(const View& v, int u, int M, int budget, const SelectLds& s, const SelectExact& ex,
                                   bool first_ready = false) {
  const int tid = threadIdx.x, lane = tid & 63;
  const size_t cb = (size_t)u * v.Mcap;
  unsigned long long* ck = (unsigned long long*)s.region;       // (score << kIdBits) | (kIdMask - id): larger goes first
  int* cw = (int*)(s.region + CMAX * 8);
#define DYNAKV_WEIGHT(j) (s.sw ? s.sw[j] : v.csz[cb + (j)])
#define DYNAKV_KEY(j) (s.skey ? s.skey[j] : orderable(v.score[cb + (j)]))
  auto key_at = [&](int j) __attribute__((always_inline)) { return DYNAKV_KEY(j); };
  // keys, sizes and the active set's bitmap in LDS: nothing is ranked, the list follows the cluster ids (emit_by_id)
  const bool id_order = s.skey && s.sw && s.selbits && M <= MAXR * NT;
  if (!first_ready) {
    for (int i = tid; i < 1024; i += NT) s.hist[i] = 0;
    if (tid < 8) s.misc[tid] = tid == 4 ? 0x7fffffff : 0;
    lds_barrier();
  }

  uint32_t kstar = 0, mask = 0;
  int above = 0, total = 0;
  bool cross = true;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    int* h = s.hist + 256 * pass;
    if (pass > 0 || !first_ready) {
      for_each_key<NT>(M, key_at, [&](int j, uint32_t k) __attribute__((always_inline)) {
        if ((k & mask) == kstar) {
          const int w = DYNAKV_WEIGHT(j);
          if (w) atomicAdd(&h[(k >> shift) & 255], w);
        }
      });
      lds_barrier();
    }
    // every wavefront: lane l owns the digits 255 - 4l .. 252 - 4l, highest first
    int hv[4], t = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) { hv[k] = h[255 - (4 * lane + k)]; t += hv[k]; }
    const int inc = wave_incl_scan(t);
    int run = above + inc - t, dstar = -1, ab = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (dstar < 0 && run + hv[k] > budget) { dstar = 255 - (4 * lane + k); ab = run; }
      run += hv[k];
    }
    const unsigned long long bal = __ballot(dstar >= 0);
    if (bal == 0) {                      // everything fits (first pass only)
      cross = false;
      total = __builtin_amdgcn_readlane(run, 63);
      break;
    }
    const int src = __ffsll((long long)bal) - 1;       // wavefront-uniform
    kstar |= (uint32_t)__builtin_amdgcn_readlane(dstar, src) << shift;
    mask |= 255u << shift;
    above = __builtin_amdgcn_readlane(ab, src);
  }

  // ---- the band around the cut, retaken in float64
  bool refined = false;
  uint32_t klo = 0, khi = 0;
  int* const band = s.hist;                             // [kBandMax] ids; the histograms are dead
  int* const bsz = s.hist + kBandMax;                   // [kBandMax] their sizes
  int* const bmask = s.hist + 2 * kBandMax;             // [2] which of them are selected
  double* const bex = (double*)(s.hist + 2 * kBandMax + 2);   // [kBandMax] their exact scores
  if (cross && ex.eps > 0.f) {
    lds_barrier();                                    // every wavefront has read the last histogram
    const float astar = unorderable(kstar);
    klo = orderable(astar - 2.f * ex.eps); khi = orderable(astar + 2.f * ex.eps);
    for_each_key<NT>(M, key_at, [&](int j, uint32_t k) __attribute__((always_inline)) {
      if (k >= klo && k <= khi) {
        const int pos = atomicAdd(&s.misc[7], 1);
        const int w = DYNAKV_WEIGHT(j);
        if (pos < kBandMax) { band[pos] = j; bsz[pos] = w; }
        if (k > kstar && w) atomicAdd(&s.misc[5], w);
      }
    });
    lds_barrier();
    const int nb = s.misc[7];
    refined = nb > 1 && nb <= kBandMax;
    if (refined) {
      if (tid < 64) {
        const uint16_t* Rq = unit_Rq(v, u);
        for (int base = 0; base < nb; base += 16) {       // four lanes per cluster, 16 clusters at a time
          const int m = base + (lane >> 2);
          const double e = quad_exact_score(v, Rq, ex.Q, u, band[min(m, nb - 1)], lane & 3);
          if ((lane & 3) == 0 && m < nb) bex[m] = e;
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_wave_barrier();
        asm volatile("" ::: "memory");
        const bool have = lane < nb;
        const double e = have ? bex[lane] : 0.0;
        const int jm = have ? band[lane] : 0x7fffffff, szm = have ? bsz[lane] : 0;
        int rank = 0, cum = above - s.misc[5];            // sizes of everything above the band
        for (int k = 0; k < nb; ++k) {
          const double ek = bex[k];
          const int jk = band[k];
          if (ek > e || (ek == e && jk < jm)) { ++rank; cum += bsz[k]; }
        }
        int rstar = have && cum + szm > budget ? rank : nb;    // rank of the first cluster that does not fit
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) rstar = min(rstar, __shfl_xor(rstar, o));
        const bool selb = have && rank < rstar;
        const unsigned long long mask = __ballot(selb);
        int tsb = selb ? szm : 0;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) tsb += __shfl_xor(tsb, o);
        if (have && rank == 0) s.misc[4] = jm;            // the best of the band: cut to the budget if nothing fits
        if (lane == 0) {
          bmask[0] = (int)(unsigned)mask; bmask[1] = (int)(unsigned)(mask >> 32);
          s.misc[5] = above - s.misc[5] + tsb;            // entries selected in all
          count(v, u, 7, 1);
        }
      }
      lds_barrier();
    }
  }

  // candidates: every score above kstar; the clusters at kstar are counted and resolved below
  for_each_key<NT>(M, key_at, [&](int j, uint32_t k) __attribute__((always_inline)) {
    if (refined && k >= klo && k <= khi) {               // a cluster of the band: its float64 decision
      bool sel = false;
      const int nb = s.misc[7];
      for (int i = 0; i < nb; ++i)
        if (band[i] == j) sel = (((unsigned)bmask[i >> 5]) >> (i & 31)) & 1u;
      v.in_req[cb + j] = sel;
      if (sel) {
        if (s.selbits) atomicOr(&s.selbits[j >> 5], 1u << (j & 31));
        if (id_order) s.misc[2] = 1;                        // (something is selected)
        else {
          const int pos = atomicAdd(&s.misc[2], 1);
          if (pos < CMAX) { ck[pos] = ((unsigned long long)k << kIdBits) | (unsigned)(kIdMask - j); cw[pos] = DYNAKV_WEIGHT(j); }
        }
      }
    } else if (cross && !refined && k == kstar) {
      atomicAdd(&s.misc[3], 1);
      atomicMin(&s.misc[4], j);
    } else {
      const bool sel = !cross || k > kstar;
      v.in_req[cb + j] = sel;
      if (sel) {
        if (s.selbits) atomicOr(&s.selbits[j >> 5], 1u << (j & 31));
        if (id_order) s.misc[2] = 1;                        // (something is selected)
        else {
          const int pos = atomicAdd(&s.misc[2], 1);
          if (pos < CMAX) { ck[pos] = ((unsigned long long)k << kIdBits) | (unsigned)(kIdMask - j); cw[pos] = DYNAKV_WEIGHT(j); }
        }
      }
    }
  });
  lds_barrier();
  int xid = s.misc[4], tie_w = 0;        // xid: the cluster at which the budget is first exceeded
  if (cross && !refined && s.misc[3] > 1) {          // several equal scores at the cut: by ascending id while they fit
    if (tid < 64) {
      int cum = above, x = -1;
      for (int base = 0; base < M && x < 0; base += 64) {
        const int j = base + lane;
        const bool tie = j < M && DYNAKV_KEY(j) == kstar;
        const int w = tie ? DYNAKV_WEIGHT(j) : 0;
        int inc = w;
        for (int o = 1; o < 64; o <<= 1) {
          const int y = __shfl_up(inc, o);
          if (lane >= o) inc += y;
        }
        const unsigned long long ob = __ballot(tie && cum + inc > budget);
        if (ob) {
          const int xl = __ffsll((long long)ob) - 1;
          x = base + xl;
          cum += __shfl(inc - w, xl);
        } else {
          cum += __shfl(inc, 63);
        }
      }
      if (lane == 0) { s.misc[4] = x < 0 ? M : x; s.misc[5] = cum - above; }
    }
    lds_barrier();
    xid = s.misc[4]; tie_w = s.misc[5];
    for (int j = tid; j < M; j += NT)
      if (DYNAKV_KEY(j) == kstar) {
        const bool sel = j < xid;
        v.in_req[cb + j] = sel;
        if (sel) {
          if (s.selbits) atomicOr(&s.selbits[j >> 5], 1u << (j & 31));
          if (id_order) s.misc[2] = 1;
          else {
            const int pos = atomicAdd(&s.misc[2], 1);
            if (pos < CMAX) { ck[pos] = ((unsigned long long)kstar << kIdBits) | (unsigned)(kIdMask - j); cw[pos] = DYNAKV_WEIGHT(j); }
          }
        }
      }
    lds_barrier();
  } else if (cross && !refined && tid == 0) {
    v.in_req[cb + xid] = 0;
  }
  if (id_order) {
    const bool truncated = cross && s.misc[2] == 0 && budget > 0;    // the best cluster alone is over budget: its first entries
    if (truncated) {
      __syncthreads();                                 // (another thread may have cleared the same active-set flag)
      if (tid == 0) {
        v.in_req[cb + xid] = 1;
        atomicOr(&s.selbits[xid >> 5], 1u << (xid & 31));
      }
      lds_barrier();
    }
    return emit_by_id<NT, MAXR>(v, u, M, s, truncated ? budget : -1);
  }
  int cut = s.misc[2], tsel = !cross ? total : refined ? s.misc[5] : above + tie_w;
  if (cut > CMAX) {
    __syncthreads();
    // keys are not in LDS (more than kSelectLds clusters) and more clusters are selected than can be ordered:
    // the retrieval is cut short to the CMAX candidates at hand and the unit's error word says so
    if (tid == 0) atomicOr(&v.err[u], DYNAKV_ERR_SELECT);
    cut = CMAX;
    tsel = -1;                                          // recomputed from the sizes below
  }
  if (cross && cut == 0 && budget > 0) {           // the best cluster alone is over budget: its first entries
    __syncthreads();                                 // (another thread may have cleared the same active-set flag)
    if (tid == 0) {
      ck[0] = ((unsigned long long)kstar << kIdBits) | (unsigned)(kIdMask - xid);
      cw[0] = budget;
      v.in_req[cb + xid] = 1;
      if (s.selbits) atomicOr(&s.selbits[xid >> 5], 1u << (xid & 31));
    }
    lds_barrier();
    cut = 1; tsel = budget;
  }

  // rank of every selected cluster = number of selected clusters that precede it.  While the workgroup has
  // several threads per selected cluster, `tpc` adjacent lanes share one cluster's count (and the first of them
  // goes on as its owner).
  constexpr int PER = (CMAX + NT - 1) / NT;
  int tpc = 1, tsh = 0;
  while (tpc < 8 && cut * tpc * 2 <= NT) { tpc <<= 1; ++tsh; }
  // Many selected clusters: counting against all of them costs cut^2 LDS reads; they are binned first
  // (bin_candidates), and a cluster's rank is the number of clusters in higher bins plus those of its own bin that
  // precede it (the sizes in s.sw, which s.srt may alias, are not read any more).
  const bool binned = cut > 256;
  int* const lst = s.srt;
  int bin_shift = 0;
  if (__builtin_expect(binned, 0)) {
    tpc = 1; tsh = 0;
    bin_shift = bin_candidates<NT>(s.hist, s.misc, lst, ck, cut);
  }
  const int sub = tid & (tpc - 1);
  const int chunk = ((cut + tpc - 1) / tpc + 7) & ~7;
  int rk[PER], idw[PER], wt[PER], pg[PER][kInlinePages];
#pragma unroll
  for (int r = 0; r < PER; ++r) {
    const int p = r == 0 ? tid >> tsh : tid + r * NT;
    rk[r] = -1; idw[r] = 0; wt[r] = 0;
#pragma unroll
    for (int k = 0; k < kInlinePages; ++k) pg[r][k] = -1;
    if (p < cut && (r == 0 || tpc == 1)) {              // wavefront-uniform per group of tpc lanes
      const unsigned long long my = ck[p];
      {   // the cluster's page table is requested now and used once its place in the list is known
        const int id = kIdMask - (int)(my & kIdMask);
        const int4* row = (const int4*)&v.cpg[(cb + id) * kInlinePages];
        const int4 a = row[0];
        pg[r][0] = a.x; pg[r][1] = a.y; pg[r][2] = a.z; pg[r][3] = a.w;
        if (cw[p] > 4 * kPageTokens) {
          const int4 b = row[1];
          pg[r][4] = b.x; pg[r][5] = b.y; pg[r][6] = b.z; pg[r][7] = b.w;
        }
      }
      int rank = 0;
      if (__builtin_expect(binned, 0)) {
        const int d = ((uint32_t)(my >> kIdBits) >> bin_shift) & 255u;
        const int b0 = s.hist[256 + d], b1 = b0 + s.hist[d];
        rank = b0;
        for (int q = b0; q < b1; ++q) rank += ck[lst[q]] > my ? 1 : 0;
      } else {
        const int q0 = r == 0 ? sub * chunk : 0, q1 = r == 0 ? min(cut, q0 + chunk) : cut;
        for (int qb = q0; qb < q1; qb += 8) {           // eight candidates per round trip to LDS
          unsigned long long o[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) o[i] = ck[min(qb + i, cut - 1)];
#pragma unroll
          for (int i = 0; i < 8; ++i) rank += (qb + i < q1 && o[i] > my) ? 1 : 0;
        }
      }
      if (r == 0) {                                     // sum over the tpc (1, 2, 4 or 8) adjacent lanes of the cluster
        if (tpc > 1) rank += dpp_or_zero<kDppXor1>(rank);
        if (tpc > 2) rank += dpp_or_zero<kDppXor2>(rank);
        if (tpc > 4) rank += dpp_or_zero<kDppHalfMirror>(rank);
      }
      if (r != 0 || sub == 0) { rk[r] = rank; idw[r] = kIdMask - (int)(my & kIdMask); wt[r] = cw[p]; }
    }
  }
  lds_barrier();
  int* by_id = cw;                 // from here on indexed by rank
  int* by_w = s.srt;
#pragma unroll
  for (int r = 0; r < PER; ++r)
    if (rk[r] >= 0) {
      by_id[rk[r]] = idw[r];
      by_w[rk[r]] = wt[r];
      v.sel_ids[cb + rk[r]] = idw[r];
    }
  lds_barrier();
  // gather offsets in rank order: running sums of the sizes (low half) and of the list entries (high half)
  unsigned long long loc[PER], run = 0;
#pragma unroll
  for (int k = 0; k < PER; ++k) {
    const int r = tid * PER + k;
    const unsigned w = r < cut ? (unsigned)by_w[r] : 0u;
    loc[k] = (unsigned long long)w | ((unsigned long long)((w + 3) >> 2) << 32);
    run += loc[k];
  }
  unsigned long long total64;
  unsigned long long pre = block_excl_scan64<true>(run, (unsigned long long*)s.sm, total64);
#pragma unroll
  for (int k = 0; k < PER; ++k) {
    const int r = tid * PER + k;
    if (r < cut)      // id, first gather offset, first list entry
      ck[r] = ((unsigned long long)by_id[r] << 46) | ((pre & 0xFFFFFFu) << 22) | ((pre >> 32) & 0x3FFFFFu);   // 18 + 24 + 22 bits
    pre += loc[k];
  }
  const int quads = tid == 0 ? (int)(total64 >> 32) : 0;
  if (tsel < 0) tsel = (int)(total64 & 0xFFFFFFFFull);
  lds_barrier();
  // list entries, by the thread that ranked the cluster (every page but the last is full, so a page's place in
  // the list follows from its index); pages past the inline table are found by walking the chain
  int* plist = v.plist + (size_t)u * v.Lcap;
  int* poff = v.plist_off + (size_t)u * v.Lcap;
#pragma unroll
  for (int r = 0; r < PER; ++r) {
    if (rk[r] < 0) continue;
    const unsigned long long pk = ck[rk[r]];
    const int t0 = (int)(pk >> 22) & 0xFFFFFF, q0 = (int)pk & 0x3FFFFF;
    const int take = wt[r], npages = (take + kPageTokens - 1) / kPageTokens;
    int page = -1;
#pragma unroll
    for (int k = 0; k < kInlinePages; ++k)
      if (k < npages) {
        page = pg[r][k];
        if (page >= 0)
          emit_page(page, min(kPageTokens, take - k * kPageTokens), q0 + 4 * k, t0 + k * kPageTokens, plist, poff,
                    s.list, s.list_cap);
      }
    for (int kk = kInlinePages; kk < npages && page >= 0; ++kk) {
      page = v.pnext[(size_t)u * v.Pcap + page];
      if (page >= 0)
        emit_page(page, min(kPageTokens, take - kk * kPageTokens), q0 + 4 * kk, t0 + kk * kPageTokens, plist, poff,
                  s.list, s.list_cap);
    }
  }
  if (quads) atomicAdd(&s.misc[6], quads);
  lds_barrier();
  const int nlist = s.misc[6];
  if (tid == 0) {
    v.n_sel[u] = cut; v.t_sel[u] = tsel; v.n_list[u] = nlist; v.ticket[u] = 0;
    count(v, u, 4, tsel);
    count(v, u, 5, 1);
    count(v, u, 6, M);
  }
#undef DYNAKV_WEIGHT
#undef DYNAKV_KEY
  return nlist;
}

// Bound on |float32 score - exact score| of a unit: float32 accumulation of 128 exact products, scaled.
__device__ inline float score_eps(const View& v, float qbound, float rmax2) {
  return kAccBound * v.scale_f * qbound * __builtin_sqrtf(rmax2) * 1.0002f * 1.01f;
}

// One workgroup per unit.  BIG: more than kSelectLds clusters per unit: scores and sizes stay in the workspace (they
// are a few hundred KB per unit and sit in L2 after the score kernel) and are read in every pass; the LDS goes to
// a larger candidate list instead.
constexpr int kCountBig = 4096;
template <bool BIG>
__global__ __launch_bounds__(1024) void select_kernel(View v, const void* Q, int budget) {
  constexpr int CMAX = BIG ? kCountBig : kCountMax;
  constexpr int kRegion = CMAX * 12;
  __shared__ uint32_t skey_[BIG ? 1 : kSelectLds];
  __shared__ __align__(16) int ssz_[BIG ? 1 : kSelectLds];   // cluster sizes: every pass of the selection reads them
  __shared__ unsigned selbits_[BIG ? 1 : kSelectLds / 32];   // the active set, one bit per cluster
  __shared__ __align__(16) unsigned char region[kRegion];
  __shared__ __align__(16) int hist[1024];
  __shared__ __align__(16) int sm[64];
  __shared__ int misc[8];
  __shared__ float qn[16];
  __shared__ int srt[CMAX];
  static_assert(kRegion >= CMAX * 12, "candidate arrays must fit");
  const int u = blockIdx.x, tid = threadIdx.x;
  const int M = v.M[u];
  if constexpr (!BIG) {
    int Mpad = 2;
    while (Mpad < M) Mpad <<= 1;
    for (int i = tid; i < Mpad; i += 1024) {
      skey_[i] = i < M ? orderable(v.score[(size_t)u * v.Mcap + i]) : 0u;
      if (i < M) ssz_[i] = v.csz[(size_t)u * v.Mcap + i];
    }
    for (int i = tid; i < kSelectLds / 32; i += 1024) selbits_[i] = 0u;
  }
  // |q_g| of every head, one wavefront per head (only where the scores came from the matrix cores)
  SelectExact ex{0.f, Q};
  if (!v.search_mean) {
    const int g = tid >> 6, lane = tid & 63;
    if (g < v.G) {
      const float a = load_elem(Q, ((size_t)u * v.G + g) * kHeadDim + lane, v.dtype);
      const float b = load_elem(Q, ((size_t)u * v.G + g) * kHeadDim + 64 + lane, v.dtype);
      float s2 = a * a + b * b;
      for (int o = 32; o > 0; o >>= 1) s2 += __shfl_xor(s2, o);
      if (lane == 0) qn[g] = __builtin_sqrtf(s2) * 1.0001f;
    }
  }
  __syncthreads();
  if (!v.search_mean) {
    float qb = 0.f;
    for (int g = 0; g < v.G; ++g) qb = v.group_reduce == DYNAKV_GROUP_MAX ? fmaxf(qb, qn[g]) : qb + qn[g];
    ex.eps = score_eps(v, qb, __int_as_float(v.rmax2[u]));
  }
  const SelectLds s{BIG ? nullptr : skey_, BIG ? nullptr : ssz_, region, hist, srt, sm, misc, nullptr, 0, BIG ? nullptr : selbits_};
  select_phase<1024, CMAX, BIG ? 8 : kSelectLds / 1024>(v, u, M, budget, s, ex);
}

// ------------------------------------------------------------------------------------------- attention
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef short s4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

// One tile of the attention loop: 16 token slots filled from up to four gather-list entries (quads), which may
// come from four different pages.  Lane l loads pieces of the K row and of the V row of token slot l % 16
// (entry slot / 4, row slot % 4 of that quad): K feeds QK^T as loaded; PV wants the four tokens of quad l / 16 of
// one column in a lane, so the V rows go through a per-wavefront LDS tile (rows padded to kVRow bytes) and come
// back transposed.  Both K and V traffic therefore follow the valid tokens exactly.
constexpr int kVRow16 = kHeadDim * 2 + 16, kVRow32 = kHeadDim * 4 + 16;   // bytes; the pad spreads the quads over the banks
constexpr int kVTile16 = kPageTokens * kVRow16, kVTile32 = kPageTokens * kVRow32;
struct Tile {
  const char* k;     // this lane's first 16 bytes of its token's K row (further pieces 64 bytes apart); the V row
                     // of the same token lies one K region further
  bool kok;          // the lane's token slot holds a token
  int nvq;           // valid tokens in the lane's PV quad (0: no entry)
};
// eK, eV: list entries of the lane's QK slot and of its PV quad (-1: none); ES = bytes per element.
template <int ES>
__device__ __forceinline__ Tile make_tile(const char* pages, int eK, int eV, int lane) {
  constexpr size_t kPageBytes = (size_t)kPageElems * ES;
  Tile t;
  t.kok = eK >= 0 && (lane & 3) <= (eK & 3);
  if (eK < 0) eK = 0;
  t.k = pages + (size_t)(eK >> 4) * kPageBytes + (((eK >> 2) & 3) * 4 + (lane & 3)) * (kHeadDim * ES) + (lane >> 4) * 16;
  t.nvq = eV >= 0 ? (eV & 3) + 1 : 0;
  return t;
}

// Fragments of one tile and of the query group, per storage type.  qk() returns S^T[token 4*(lane/16)+i]
// [head lane%16]; pv() adds P^T-weighted V^T into acc[cb][i] = O^T[column out_col(cb, 4*(lane/16) + i)][head lane%16].
template <int DT>
struct Frag;

template <>
struct Frag<DYNAKV_F32> {
  struct KV { f4 k[8]; f4 v[8]; };     // v: this lane's pieces of its token's V row, as loaded
  struct VT { f4 c[8]; };              // c[cb][kk] = V[token 4*(lane/16) + kk][column out_col(cb, lane%16)]
  struct Qf { f4 b[8]; };
  static constexpr int kVTile = kVTile32;
  static __device__ __forceinline__ void load_q(Qf& q, const void* Q, size_t row, int lg, bool ok) {
    const float* p = (const float*)Q + row * kHeadDim + 4 * lg;
#pragma unroll
    for (int s = 0; s < 8; ++s) q.b[s] = ok ? *(const f4*)(p + 16 * s) : f4{0, 0, 0, 0};
  }
  static __device__ __forceinline__ void load(KV& f, const Tile& t) {
    const f4* kp = (const f4*)t.k;
    const f4* vp = (const f4*)(t.k + 2048 * 4);
#pragma unroll
    for (int s = 0; s < 8; ++s) f.k[s] = t.kok ? kp[s * 4] : f4{0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 8; ++s) f.v[s] = t.kok ? vp[s * 4] : f4{0, 0, 0, 0};
  }
  // V rows -> LDS tile of this wavefront (zeros for empty slots), then back with tokens innermost
  static __device__ __forceinline__ void stage(const KV& f, char* tile, int lane) {
    char* row = tile + (lane & 15) * kVRow32 + (lane >> 4) * 16;
#pragma unroll
    for (int s = 0; s < 8; ++s) *(f4*)(row + s * 64) = f.v[s];
  }
  static __device__ __forceinline__ int out_col(int cb, int a) { return 16 * cb + a; }   // row a of accumulator block cb
  static __device__ __forceinline__ void unstage(VT& t, const char* tile, int lane) {
    const char* p = tile + (lane >> 4) * 4 * kVRow32 + (lane & 15) * 4;
#pragma unroll
    for (int cb = 0; cb < 8; ++cb)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) t.c[cb][kk] = *(const float*)(p + kk * kVRow32 + cb * 64);
  }
  static __device__ __forceinline__ f4 qk(const KV& f, const Qf& q) {
    f4 a = {0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int i = 0; i < 4; ++i) a = __builtin_amdgcn_mfma_f32_16x16x4f32(f.k[s][i], q.b[s][i], a, 0, 0, 0);
    return a;
  }
  static __device__ __forceinline__ void pv(f4 (&acc)[8], const VT& f, const float (&p)[4]) {
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(f.c[c][kk], p[kk], acc[c], 0, 0, 0);
  }
};

template <bool BF>
struct Frag16 {
  struct KV { uint4 k[4]; uint4 v[4]; };   // v: this lane's pieces of its token's V row, as loaded
  struct VT { uint2 c[8]; };               // c[cb] = V[tokens 4*(lane/16) .. +3][column out_col(cb, lane%16)]
  struct Qf { uint4 b[4]; };
  static constexpr int kVTile = kVTile16;
  static __device__ __forceinline__ void load_q(Qf& q, const void* Q, size_t row, int lg, bool ok) {
    const uint16_t* p = (const uint16_t*)Q + row * kHeadDim + 8 * lg;
#pragma unroll
    for (int s = 0; s < 4; ++s) q.b[s] = ok ? *(const uint4*)(p + 32 * s) : uint4{0, 0, 0, 0};
  }
  static __device__ __forceinline__ void load(KV& f, const Tile& t) {
    const uint4* kp = (const uint4*)t.k;
    const uint4* vp = (const uint4*)(t.k + 2048 * 2);
#pragma unroll
    for (int s = 0; s < 4; ++s) f.k[s] = t.kok ? kp[s * 4] : uint4{0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 4; ++s) f.v[s] = t.kok ? vp[s * 4] : uint4{0, 0, 0, 0};
  }
  // V rows -> LDS tile of this wavefront (zeros for empty slots), then back with tokens innermost
  static __device__ __forceinline__ void stage(const KV& f, char* tile, int lane) {
    char* row = tile + (lane & 15) * kVRow16 + (lane >> 4) * 16;
#pragma unroll
    for (int s = 0; s < 4; ++s) *(uint4*)(row + s * 64) = f.v[s];
  }
  // row a of accumulator block cb is this output column: a lane reads column pairs (one 32-bit word per token)
  static __device__ __forceinline__ int out_col(int cb, int a) { return 32 * (cb >> 1) + 2 * a + (cb & 1); }
  static __device__ __forceinline__ void unstage(VT& t, const char* tile, int lane) {
    const char* p = tile + (lane >> 4) * 4 * kVRow16 + (lane & 15) * 4;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      uint32_t w[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) w[kk] = *(const uint32_t*)(p + kk * kVRow16 + s * 64);
      t.c[2 * s] = uint2{(w[0] & 0xffffu) | (w[1] << 16), (w[2] & 0xffffu) | (w[3] << 16)};
      t.c[2 * s + 1] = uint2{(w[0] >> 16) | (w[1] & 0xffff0000u), (w[2] >> 16) | (w[3] & 0xffff0000u)};
    }
  }
  static __device__ __forceinline__ f4 qk(const KV& f, const Qf& q) {
    f4 a = {0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if constexpr (BF)
        a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, f.k[s]), __builtin_bit_cast(b8, q.b[s]), a, 0, 0, 0);
      else
        a = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, f.k[s]), __builtin_bit_cast(h8, q.b[s]), a, 0, 0, 0);
    }
    return a;
  }
  static __device__ __forceinline__ f4 mma4(uint2 a, uint2 b, f4 c) {
    if constexpr (BF)
      return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s4, a), __builtin_bit_cast(s4, b), c, 0, 0, 0);
    else
      return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(h4, a), __builtin_bit_cast(h4, b), c, 0, 0, 0);
  }
  // p is split into a rounded part and its remainder so that the product keeps float32-like accuracy
  static __device__ __forceinline__ void pv(f4 (&acc)[8], const VT& f, const float (&p)[4]) {
    uint16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if constexpr (BF) {
        const __bf16 h = (__bf16)p[i];
        const __bf16 l = (__bf16)(p[i] - (float)h);
        hi[i] = __builtin_bit_cast(uint16_t, h);
        lo[i] = __builtin_bit_cast(uint16_t, l);
      } else {
        const _Float16 h = (_Float16)p[i];
        const _Float16 l = (_Float16)(p[i] - (float)h);
        hi[i] = __builtin_bit_cast(uint16_t, h);
        lo[i] = __builtin_bit_cast(uint16_t, l);
      }
    }
    const uint2 ph = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
    const uint2 pl = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      acc[c] = mma4(f.c[c], ph, acc[c]);
      acc[c] = mma4(f.c[c], pl, acc[c]);
    }
  }
};
template <> struct Frag<DYNAKV_F16> : Frag16<false> {};
template <> struct Frag<DYNAKV_BF16> : Frag16<true> {};

// Merges `n` partial results (running max in the log2 domain, denominator, one accumulator) that sit
// `stride` floats apart.  DEVICE: the partial results were written by other workgroups (see st_device).
template <bool DEVICE = false>
__device__ inline void merge_partials(const float* mx, const float* den, const float* acc, int n, int stride,
                                      float& M, float& L, float& O) {
  auto ld = [](const float* p) {
    return DEVICE ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
  };
  M = -__builtin_inff();
  for (int w = 0; w < n; ++w) M = fmaxf(M, ld(mx + (size_t)w * stride));
  L = 0.f; O = 0.f;
  for (int w = 0; w < n; ++w) {
    const float mw = ld(mx + (size_t)w * stride);
    if (mw == -__builtin_inff()) continue;
    const float sc = __builtin_amdgcn_exp2f(mw - M);
    L += sc * ld(den + (size_t)w * stride);
    O += sc * ld(acc + (size_t)w * stride);
  }
}
// Store that other workgroups of the device can read back (with the matching load above) once it has completed,
// without any cache-wide write-back or invalidation: both go past the caches that are not coherent across the
// chip.  A device-scope fence would do the same for all memory at a cost that grows with every workgroup.
__device__ inline void st_device(float* p, float x) { __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Per-wavefront running state of the online softmax.
struct Softmax {
  float m, l;
  f4 acc[8];
};

// One tile: S^T = K Q^T on the matrix cores, running max / rescale, O^T += V^T P^T.
template <class F>
__device__ __forceinline__ void consume_page(Softmax& st, const typename F::KV& kv, const typename F::Qf& q, int nvq, float sc,
                                    char* vtile, int lane) {
  F::stage(kv, vtile, lane);              // the scores are computed while the V rows settle in LDS
  const f4 sacc = F::qk(kv, q);
  float s2[4], mx = -__builtin_inff();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    s2[i] = i < nvq ? sacc[i] * sc : -__builtin_inff();
    mx = fmaxf(mx, s2[i]);
  }
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float mn = fmaxf(st.m, mx);          // finite: every tile has a valid token
  const float alpha = __builtin_amdgcn_exp2f(st.m - mn);
  float pr[4], ps = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) { pr[i] = __builtin_amdgcn_exp2f(s2[i] - mn); ps += pr[i]; }
  st.l = st.l * alpha + ps;
  st.m = mn;
#pragma unroll
  for (int c = 0; c < 8; ++c) st.acc[c] *= alpha;
  asm volatile("" ::: "memory");          // same wavefront: LDS keeps program order, the compiler must too
  typename F::VT vt;
  F::unstage(vt, vtile, lane);
  asm volatile("" ::: "memory");
  F::pv(st.acc, vt, pr);
}

// grid (S, U); NW wavefronts per workgroup; the unit's gather list is dealt tile by tile (four entries) to the
// S * NW wavefronts.  Each wavefront first fetches the entries of its next 16 tiles with one gathered load
// (lane l holds entry l % 4 of tile l / 4), so page addresses never wait on a dependent load inside the loop;
// with PF the next tile's loads are issued before the current tile is consumed.
template <int DT, int NW, bool PF>
__global__ __launch_bounds__(NW * 64) void gather_attend_kernel(View v, const void* Q, float* out, float* lse) {
  using F = Frag<DT>;
  constexpr int ES = DT == DYNAKV_F32 ? 4 : 2;
  // one V tile per wavefront during the loop, then [NW][G][130]: accumulators, max, denominator per wave and head
  extern __shared__ __align__(16) float sm_o[];
  __shared__ int s_last;
  const int u = blockIdx.y, s = blockIdx.x, S = gridDim.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane & 15, lg = lane >> 4, G = v.G;

  typename F::Qf q;
  F::load_q(q, Q, (size_t)u * G + (g < G ? g : 0), lg, g < G);
  const int nlist = v.n_list[u], ntile = (nlist + 3) >> 2;
  const int* plist = v.plist + (size_t)u * v.Lcap;
  const char* pages = v.pages + (size_t)u * v.Pcap * kPageElems * ES;
  const float sc = v.scale_f * kLog2e;

  Softmax st;
  st.m = -__builtin_inff(); st.l = 0.f;
#pragma unroll
  for (int c = 0; c < 8; ++c) st.acc[c] = f4{0, 0, 0, 0};

  const int stride = S * NW, p0 = s * NW + wave;
  const int mine = p0 < ntile ? (ntile - p0 + stride - 1) / stride : 0;   // tiles of this wavefront
  const int selK = (lane & 15) >> 2;
  char* vtile = (char*)sm_o + wave * F::kVTile;
  for (int c0 = 0; c0 < mine; c0 += 16) {
    const int cn = min(16, mine - c0);
    const int my_e = 4 * (p0 + (c0 + (lane >> 2)) * stride) + (lane & 3);
    const int e_l = (lane >> 2) < cn && my_e < nlist ? plist[my_e] : -1;
    if constexpr (PF) {
      typename F::KV a, b;
      Tile ta = make_tile<ES>(pages, __shfl(e_l, selK), __shfl(e_l, lg), lane), tb = ta;
      F::load(a, ta);
      for (int i = 0; i < cn; i += 2) {
        if (i + 1 < cn) {
          tb = make_tile<ES>(pages, __shfl(e_l, 4 * (i + 1) + selK), __shfl(e_l, 4 * (i + 1) + lg), lane);
          F::load(b, tb);
        }
        consume_page<F>(st, a, q, ta.nvq, sc, vtile, lane);
        if (i + 1 < cn) {
          if (i + 2 < cn) {
            ta = make_tile<ES>(pages, __shfl(e_l, 4 * (i + 2) + selK), __shfl(e_l, 4 * (i + 2) + lg), lane);
            F::load(a, ta);
          }
          consume_page<F>(st, b, q, tb.nvq, sc, vtile, lane);
        }
      }
    } else {
      for (int i = 0; i < cn; ++i) {
        typename F::KV a;
        const Tile ta = make_tile<ES>(pages, __shfl(e_l, 4 * i + selK), __shfl(e_l, 4 * i + lg), lane);
        F::load(a, ta);
        consume_page<F>(st, a, q, ta.nvq, sc, vtile, lane);
      }
    }
  }
  float l = st.l;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  // workgroup merge
  __syncthreads();                                    // the V tiles are dead: their space becomes the merge buffer
  const int hs = kHeadDim + 2, ws = G * hs;
  if (g < G) {
    float* o = sm_o + wave * ws + g * hs;
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) o[F::out_col(c, 4 * lg + i)] = st.acc[c][i];
    if (lg == 0) { o[kHeadDim] = st.m; o[kHeadDim + 1] = l; }
  }
  __syncthreads();
  float* part = v.part + ((size_t)u * S + s) * ws;
  for (int t = threadIdx.x; t < G * kHeadDim; t += NW * 64) {
    const int gg = t / kHeadDim, dc = t % kHeadDim;
    const float* b = sm_o + gg * hs;
    float M, L, O;
    merge_partials(b + kHeadDim, b + kHeadDim + 1, b + dc, NW, ws, M, L, O);
    if (S == 1) {
      out[((size_t)u * G + gg) * kHeadDim + dc] = L > 0.f ? O / L : 0.f;
      if (lse && dc == 0) lse[(size_t)u * G + gg] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * kLn2 : -__builtin_inff();
    } else {
      st_device(&part[gg * hs + dc], O);
      if (dc == 0) { st_device(&part[gg * hs + kHeadDim], M); st_device(&part[gg * hs + kHeadDim + 1], L); }
    }
  }
  if (S == 1) return;
  // the last workgroup of the unit to arrive merges all partial results: every thread waits for its own stores
  // to complete, the barrier collects the workgroup, then one thread takes the ticket
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  // release: this workgroup's partial results happen before its ticket; acquire: the last arriver sees all of them
  if (threadIdx.x == 0)
    s_last = __hip_atomic_fetch_add(&v.ticket[u], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == S - 1;
  __syncthreads();
  if (!s_last) return;
  const float* all = v.part + (size_t)u * S * ws;
  for (int t = threadIdx.x; t < G * kHeadDim; t += NW * 64) {
    const int gg = t / kHeadDim, dc = t % kHeadDim;
    const float* b = all + gg * hs;
    float M, L, O;
    merge_partials<true>(b + kHeadDim, b + kHeadDim + 1, b + dc, S, ws, M, L, O);
    out[((size_t)u * G + gg) * kHeadDim + dc] = L > 0.f ? O / L : 0.f;
    if (lse && dc == 0) lse[(size_t)u * G + gg] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * kLn2 : -__builtin_inff();
  }
}

// Whole retrieval of one unit in one workgroup (16-bit storage, at most kFusedClusters clusters and 8 query heads
// per unit; at every unit count, because the step is bound by dependent round trips rather than by the number of
// busy compute units): scores -> LDS, budget cut in LDS, gather list in LDS, then the same page loop and merge
// as gather_attend_kernel.  Saves two launches and every trip through the workspace between the phases.
constexpr int kFusedList = 2048;       // gather-list entries it keeps in LDS (longer lists are read from the workspace)

// With APPEND the same pass over the centroid table also finds the cluster nearest to the step's new key
// (one more accumulator per centroid), and the append itself is committed after the selection (the gather list is
// fixed by then and the append touches nothing it names): a decode step then reads the table once instead of
// twice.  Scores and selection see the index as it was before the append.
// With SPLIT (only with APPEND) the unit's due splits are part of the same launch: a whole decode step is then
// one kernel.  The splits are planned right after the append; while the pages are streamed, the first wavefronts,
// one per due split (up to kWaveSplits), decide their split instead of streaming, which only reads the index;
// these splits are written while the attention output is merged, and whatever is left (recycling the parents'
// pages, further splits, the workgroup-wide path for large clusters) is carried out by the first kSplitThreads
// threads, once the others have left.
template <int DT, int NW, int GP, bool APPEND, bool SPLIT>
__global__ __launch_bounds__(NW * 64) void retrieve_fused_kernel(View v, const void* Q, int budget, float* out,
                                                                float* lse, const void* kin, const void* vin) {
  using F = Frag<DT>;
  constexpr int NT = NW * 64;
  constexpr int ES = DT == DYNAKV_F32 ? 4 : 2;
  constexpr int kMergeBytes = 64 * (kHeadDim + 2) * 4;          // NW * G <= 64 head rows
  constexpr int kKeys = kFusedClusters * 4, kSizes = kFusedClusters * 4, kList = kFusedList * 4;
  static_assert(kSelRegion >= 2 * kFusedClusters && kKeys + kSizes + kSelRegion + kList >= kMergeBytes, "LDS plan");
  static_assert(NW * F::kVTile <= kKeys + kSizes + kSelRegion, "the V tiles take the space of the selection's tables");
  // scores, sizes, candidates, gather list; after the page loop the front doubles as the merge buffer
  constexpr size_t kPhases = kKeys + kSizes + kSelRegion + kList;
  static_assert(!SPLIT || (APPEND && NW * 64 >= kSplitThreads), "splits follow an append");
  // the split's LDS follows everything the streaming uses: its wavefront contexts are filled meanwhile
  constexpr int kPreSplits = kWaveSplits;              // splits decided while the pages are streamed
  constexpr size_t kRawOff = SPLIT ? (kPhases + 15) / 16 * 16 : 0;
  static_assert(!SPLIT || kRawOff + kSplitRaw + 16 * 1024 <= 160 * 1024, "LDS of one compute unit");
  __shared__ __align__(16) unsigned char smem[SPLIT ? kRawOff + kSplitRaw : kPhases];
  __shared__ SplitWork wk;
  __shared__ AppendSmem ap;
  __shared__ double am_v[16];
  __shared__ int am_i[16];
  __shared__ float am_2[16];
  __shared__ int am_r[16];
  __shared__ int s_tile;                              // next tile of the page stream
  __shared__ unsigned selbits[kFusedClusters / 32];    // the active set: for the gather list and the plan of the splits
  __shared__ __align__(16) int sm[64];
  __shared__ int misc[8];
  uint32_t* skey = (uint32_t*)smem;
  int* ssz = (int*)(smem + kKeys);
  int* list = (int*)(smem + kKeys + kSizes + kSelRegion);
  int* hist = list;                                   // the histograms are dead before the list is written
  static_assert(kList >= 1024 * 4, "histograms must fit the list");
  float* sm_o = (float*)smem;
  const int u = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int G = v.G;

  // ---- scores on the matrix cores.  Tiles of 16 clusters are dealt round-robin: wavefront w takes the tiles w,
  // w + NW, ...; kBatch of them are consumed while the loads of the next kBatch are in flight (16 KB per wavefront).
  constexpr bool BF = DT == DYNAKV_BF16;
  constexpr int kBatch = 4;
  const uint16_t* Rq = unit_Rq(v, u);
  const uint4* tiles = (const uint4*)Rq;
  const int table_tiles = (int)(v.Rstride / kTileElems);   // the table's padded end: these rows exist in every state
  uint4 cur[kBatch][4], nxt[kBatch][4];
  auto fetch = [&](uint4 (&dst)[kBatch][4], int t0) __attribute__((always_inline)) {
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      const int T = t0 + b * NW;
#pragma unroll
      for (int s2 = 0; s2 < 4; ++s2) dst[b][s2] = T < table_tiles ? tiles[((size_t)T * 4 + s2) * 64 + lane] : uint4{0, 0, 0, 0};
    }
  };
  fetch(cur, wave);                                   // requested before anything is waited for
  // the flagged list and the free-page stack as they are before this step's append: the plan of the splits
  // starts from them
  int flagged0 = 0, nflag0 = 0, top0 = 0;            // kept in LDS (wk) until the selection is done
  if constexpr (SPLIT)
    if (wave == 0) {
      if (lane < v.Mcap) flagged0 = v.flist[(size_t)u * v.Mcap + lane];
      nflag0 = v.nflag[u];
      top0 = v.free_top[u];
    }
  const int M = v.M[u];
  // stored sizes, requested for every cluster slot of the unit so that the requests do not wait for M
  int szr[kFusedClusters / NT];
#pragma unroll
  for (int k = 0; k < kFusedClusters / NT; ++k) {
    const int j = tid + k * NT;
    szr[k] = j < v.Mcap ? v.csz[(size_t)u * v.Mcap + j] : 0;
  }
  ScoreRows<1> A;
  load_score_rows<1>(A, G, Q, APPEND ? kin : nullptr, u, lane);
  const int N = APPEND ? v.N[u] : 0;
  const bool room = APPEND && N < v.Ncap;              // otherwise the append is refused, as by the append kernel
  if (APPEND && tid < kHeadDim) ap.kd[tid] = (double)load_elem(kin, (size_t)u * kHeadDim + tid, v.dtype);
  int Mpad = 2;
  while (Mpad < M) Mpad <<= 1;
  for (int i = M + tid; i < Mpad; i += NT) skey[i] = 0u;
  for (int i = tid; i < 1024; i += NT) hist[i] = 0;
  if (tid < 8) misc[tid] = tid == 4 ? 0x7fffffff : 0;
  if (tid == 0) { s_tile = 0; if constexpr (SPLIT) wk.ready = 0; }
  if (tid < kFusedClusters / 32) selbits[tid] = 0u;
#pragma unroll
  for (int k = 0; k < kFusedClusters / NT; ++k)
    if (tid + k * NT < M) ssz[tid + k * NT] = szr[k];
  if constexpr (SPLIT)
    if (wave == 0) {
      wk.flagged0[lane] = flagged0;
      if (lane == 0) { wk.nflag0 = nflag0; wk.top0 = top0; }
    }
  const RowNorms rn = row_norms<BF, 1>(A, G, v.group_reduce, lane);
  lds_barrier();
  float zb = -__builtin_inff(), z2 = -__builtin_inff(), rmax2 = 0.f;
  int jb = -1;
  const int nctile = (M + kTileClusters - 1) / kTileClusters;
  for (int t0 = wave; t0 < nctile; t0 += kBatch * NW) {
    const bool more = t0 + kBatch * NW < nctile;
    if (more) fetch(nxt, t0 + kBatch * NW);
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      const int T = t0 + b * NW;
      if (T >= nctile) break;                          // wavefront-uniform
      float red, kdot, nrm2;
      score_tile<BF, 1, APPEND>(cur[b], A, G, v.group_reduce, lane, red, kdot, nrm2);
      const int j = T * kTileClusters + lane;
      if (lane < kTileClusters && j < M) {
        const float sc = red * v.scale_f;
        v.score[(size_t)u * v.Mcap + j] = sc;
        const uint32_t key = orderable(sc);
        skey[j] = key;
        const int w = ssz[j];                          // first pass of the selection's radix search
        if (w) atomicAdd(&hist[key >> 24], w);
        rmax2 = fmaxf(rmax2, nrm2);
        if constexpr (APPEND) {
          const float z = kdot - 0.5f * nrm2;
          v.zdist[(size_t)u * v.Mcap + j] = z;
          if (jb < 0 || z > zb) { z2 = jb < 0 ? z2 : zb; zb = z; jb = j; }     // ascending j per lane: the first maximum stays
          else z2 = fmaxf(z2, z);
        }
      }
    }
    if (more) {
#pragma unroll
      for (int b = 0; b < kBatch; ++b)
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) cur[b][s2] = nxt[b][s2];
    }
  }
  // every wavefront leaves its largest |r|^2 and, for the append, its best / runner-up; one barrier, and every thread
  // combines the NW entries
  const int rm = wave_max(__float_as_int(rmax2));      // non-negative floats order like their bits
  if constexpr (APPEND) wave_best2(zb, jb, z2);
  if (lane == 0) {
    am_r[wave] = rm;
    if constexpr (APPEND) { am_v[wave] = (double)zb; am_i[wave] = jb; am_2[wave] = z2; }
  }
  lds_barrier();                                      // scores, first histogram and the wavefronts' results are in place
  int rmu = am_r[0];
#pragma unroll
  for (int k = 1; k < NW; ++k) rmu = max(rmu, am_r[k]);
  const float unit_rmax2 = __int_as_float(rmu);
  // the append's nearest cluster: its record is requested here and used after the selection
  int ja = -1;
  AppendFetchWave apf{0.0, 0.0, 0.0, 0, 0};
  if constexpr (APPEND) {
    ja = nearest_decide<NT>(v, u, M, rn.kn, unit_rmax2, v.zdist + (size_t)u * v.Mcap, Rq, ap.kd, am_v, am_i, am_2);
    if (room && wave == 0) apf = append_fetch_wave(v, u, ja);       // the first wavefront will carry out the append
  }

  // ---- selection
  const SelectLds sel{skey, ssz, smem + kKeys + kSizes, hist, ssz, sm, misc, list, kFusedList, selbits};
  const SelectExact ex{score_eps(v, rn.qbound, unit_rmax2), Q};
  const int nlist = select_phase<NT>(v, u, M, budget, sel, ex, true);
  // a full barrier only where other threads read back what the selection wrote to memory: a list too long for LDS
  // (page loop); the plan of the splits takes the active set from the bitmap in LDS
  if (nlist > kFusedList) __syncthreads();
  else lds_barrier();

  // ---- the append, the plan of the splits, and gather + attention.  Scores and selection saw the index as it was
  // before the append; the gather list is fixed, and the append touches nothing it names.  So the first wavefront
  // carries out the append and plans the step's splits on its own (no workgroup barrier) while the others already
  // stream pages.  Tiles are handed out through an LDS counter, so it does not matter who streams: once the plan is
  // known (wk.ready), the first wk.npre wavefronts turn to deciding one split each (they only read the index),
  // the first of them being the wavefront that made the plan; everybody else streams until the tiles run out.
  const int g = lane & 15, lg = lane >> 4;
  typename F::Qf q;
  F::load_q(q, Q, (size_t)u * G + (g < G ? g : 0), lg, g < G);
  const int* plist = v.plist + (size_t)u * v.Lcap;
  const char* pages = v.pages + (size_t)u * v.Pcap * kPageElems * ES;
  const float sc = v.scale_f * kLog2e;
  Softmax st;
  st.m = -__builtin_inff(); st.l = 0.f;
#pragma unroll
  for (int c = 0; c < 8; ++c) st.acc[c] = f4{0, 0, 0, 0};
  const int* src = nlist <= kFusedList ? list : plist;
  const int ntile = (nlist + 3) >> 2, selK = (lane & 15) >> 2;
  char* vtile = (char*)smem + wave * F::kVTile;            // scores, sizes and candidates are dead
  uint4 pre_v[kVAhead] = {};
  bool decides = false;                                // this wavefront decides a split instead of streaming
  if constexpr (APPEND) {
    if (wave == 0) {
      PlanEarly pe{};
      if constexpr (SPLIT) {
        flagged0 = wk.flagged0[lane]; nflag0 = wk.nflag0; top0 = wk.top0;
        pe = plan_fetch_early(v, u, flagged0, nflag0, top0, room ? ja : -1, lane, selbits);
      }
      if (room) append_commit_wave(v, u, ja, M, N, kin, vin, ap, apf);
      else if (lane == 0) v.err[u] |= DYNAKV_ERR_TOKENS;
      if constexpr (SPLIT) {
        wave_sync();
        plan_finish<DT>(v, wk, pe, nflag0, top0, M, ja, room ? &ap : nullptr, kPreSplits);
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");     // plan and appended entry before the flag
        if (lane == 0) __hip_atomic_store(&wk.ready, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        decides = wk.npre > 0;
      }
    }
  }
#define DYNAKV_TILE(T) make_tile<ES>(pages, 4 * (T) + selK < nlist ? src[4 * (T) + selK] : -1, \
                                     4 * (T) + lg < nlist ? src[4 * (T) + lg] : -1, lane)
  // next tile of the unit (wavefront-uniform); tiles past the end mean there is nothing left
  auto grab = [&]() __attribute__((always_inline)) {
    int t = 0;
    if (lane == 0) t = atomicAdd(&s_tile, 1);
    return __builtin_amdgcn_readfirstlane(t);
  };
  // a wavefront that may be asked to decide a split looks at the plan between two tiles
  auto called_away = [&]() __attribute__((always_inline)) {
    if constexpr (SPLIT) {
      if (wave > 0 && wave < kPreSplits && !decides &&
          __hip_atomic_load(&wk.ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) != 0 && wave < wk.npre)
        decides = true;
    }
    return decides;
  };
  if (!decides) {                                     // two tiles in flight per wavefront
    typename F::KV a, b;
    int p0 = called_away() ? ntile : grab(), p1;
    Tile ta = DYNAKV_TILE(min(p0, max(ntile - 1, 0))), tb = ta;
    if (p0 < ntile) F::load(a, ta);
    while (p0 < ntile) {
      p1 = called_away() ? ntile : grab();
      if (p1 < ntile) {
        tb = DYNAKV_TILE(p1);
        F::load(b, tb);
      }
      consume_page<F>(st, a, q, ta.nvq, sc, vtile, lane);
      if (p1 >= ntile) break;
      p0 = called_away() ? ntile : grab();
      if (p0 < ntile) {
        ta = DYNAKV_TILE(p0);
        F::load(a, ta);
      }
      consume_page<F>(st, b, q, tb.nvq, sc, vtile, lane);
    }
  }
#undef DYNAKV_TILE
  if constexpr (SPLIT) {
    // wavefronts 1 .. kPreSplits - 1 whose tiles ran out before the plan was there wait for it (it is a few
    // microseconds away at most: the first wavefront does nothing else first)
    if (wave > 0 && wave < kPreSplits && !decides) {
      int spins = 0;
      while (__hip_atomic_load(&wk.ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0 && ++spins < (1 << 20))
        __builtin_amdgcn_s_sleep(1);
      decides = wave < wk.npre;
    }
    if (decides) split_predecide<DT>(v, u, smem + kRawOff, wk, wave, pre_v);
  }
  float l = st.l;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  lds_barrier();                                      // the list is dead: its space becomes the merge buffer
  int nprep = 0;
  if constexpr (SPLIT) nprep = wk.npre;
  const int hs = kHeadDim + 2, ws = G * hs;
  if (g < G) {
    float* o = sm_o + wave * ws + g * hs;
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) o[F::out_col(c, 4 * lg + i)] = st.acc[c][i];
    if (lg == 0) { o[kHeadDim] = st.m; o[kHeadDim + 1] = l; }
  }
  // the splits decided meanwhile get their ids and pages in plan order (one thread) ...
  if constexpr (SPLIT)
    if (tid == 0 && nprep > 0) split_assign(v, u, (WaveCtx*)(smem + kRawOff), wk.pl, nprep);
  lds_barrier();
  if (SPLIT && wave < nprep) {
    // ... and are written by the wavefronts that decided them, while the others merge the attention output
    wave_split_commit<DT>(v, u, ((WaveCtx*)(smem + kRawOff))[ctx_of(wave)], pre_v, true);
  } else {
    for (int t = tid - nprep * 64; t < G * kHeadDim; t += NT - nprep * 64) {
      const int gg = t / kHeadDim, dc = t % kHeadDim;
      const float* b = sm_o + gg * hs;
      float Mx, L, O;
      merge_partials(b + kHeadDim, b + kHeadDim + 1, b + dc, NW, ws, Mx, L, O);
      out[((size_t)u * G + gg) * kHeadDim + dc] = L > 0.f ? O / L : 0.f;
      if (lse && dc == 0) lse[(size_t)u * G + gg] = L > 0.f ? (Mx + __builtin_amdgcn_logf(L)) * kLn2 : -__builtin_inff();
    }
  }
  if constexpr (SPLIT) {
    __syncthreads();                                 // every use of smem lies behind
    if (tid >= kSplitThreads) return;                // barriers from here on count the remaining wavefronts only
    split_unit<DT>(v, u, smem + kRawOff, wk, true);
  }
}

template <int DT, int NW, bool PF>
void launch_ga(const View& v, const void* Q, float* out, float* lse, hipStream_t st) {
  const size_t lds = std::max((size_t)NW * v.G * (kHeadDim + 2) * sizeof(float), (size_t)NW * Frag<DT>::kVTile);
  gather_attend_kernel<DT, NW, PF><<<dim3(v.S, v.U), NW * 64, lds, st>>>(v, Q, out, lse);
}
template <int DT>
void launch_ga_dt(const View& v, const void* Q, float* out, float* lse, hipStream_t st) {
  // 16 wavefronts hold one page each; fewer wavefronts keep a second page in flight instead
  switch (v.NW) {
    case 16: launch_ga<DT, 16, false>(v, Q, out, lse, st); break;
    case 8: launch_ga<DT, 8, true>(v, Q, out, lse, st); break;
    default: launch_ga<DT, 4, true>(v, Q, out, lse, st); break;
  }
}

}  // namespace

bool retrieve_is_fused(const View& v) {
  return v.fuse && v.S == 1 && !v.search_mean && !v.token_level && v.Mcap <= kFusedClusters && v.G <= 8;
}

template <int DT, bool APPEND, bool SPLIT>
static void launch_fused(const View& v, const void* Q, int budget, float* out, float* lse, const void* kin,
                         const void* vin, hipStream_t st) {
  // eight wavefronts: 256 registers per lane leave room for float64 scoring and a second tile in flight
  if (v.G <= 4) retrieve_fused_kernel<DT, 8, 4, APPEND, SPLIT><<<v.U, 512, 0, st>>>(v, Q, budget, out, lse, kin, vin);
  else retrieve_fused_kernel<DT, 8, 8, APPEND, SPLIT><<<v.U, 512, 0, st>>>(v, Q, budget, out, lse, kin, vin);
}

// kin == nullptr: retrieval only; otherwise retrieval followed by the append of (kin, vin) and, with `split`,
// by the splits that are due.
hipError_t launch_retrieve_fused(const View& v, const void* Q, int budget, float* out, float* lse, const void* kin,
                                 const void* vin, bool split, hipStream_t st) {
  if (v.dtype == DYNAKV_F16) {
    if (kin && split) launch_fused<DYNAKV_F16, true, true>(v, Q, budget, out, lse, kin, vin, st);
    else if (kin) launch_fused<DYNAKV_F16, true, false>(v, Q, budget, out, lse, kin, vin, st);
    else launch_fused<DYNAKV_F16, false, false>(v, Q, budget, out, lse, kin, vin, st);
  } else {
    if (kin && split) launch_fused<DYNAKV_BF16, true, true>(v, Q, budget, out, lse, kin, vin, st);
    else if (kin) launch_fused<DYNAKV_BF16, true, false>(v, Q, budget, out, lse, kin, vin, st);
    else launch_fused<DYNAKV_BF16, false, false>(v, Q, budget, out, lse, kin, vin, st);
  }
  return hipGetLastError();
}

// Workgroups per unit of the matrix-core score kernel: about five per compute unit over all units, each wavefront
// walking several groups of 64 clusters with the next group's rows in flight.
static dim3 score_grid(const View& v) {
  int gx = (1280 + v.U - 1) / v.U;
  gx = gx < 1 ? 1 : (gx > v.NB ? v.NB : gx);
  return dim3(gx, v.U);
}

hipError_t launch_score_select(const View& v, const void* Q, int budget, const void* kin, hipStream_t st) {
  dim3 grid((v.Mcap + 255) / 256, v.U);
  if (v.search_mean) {
#define DYNAKV_SCORE_G(GP)                                                              \
  do {                                                                                  \
    if (kin) score_mean_kernel<GP, true><<<grid, 256, 0, st>>>(v, Q, kin);              \
    else score_mean_kernel<GP, false><<<grid, 256, 0, st>>>(v, Q, nullptr);             \
  } while (0)
    if (v.G <= 4) DYNAKV_SCORE_G(4);
    else if (v.G <= 8) DYNAKV_SCORE_G(8);
    else DYNAKV_SCORE_G(16);
#undef DYNAKV_SCORE_G
  } else {
    // G query heads and, with kin, the new key: one block of 16 rows, two if that makes 17
#define DYNAKV_SCORE_B(BF, NBLK)                                                               \
  do {                                                                                         \
    if (kin) score_mfma_kernel<BF, NBLK, true, true><<<grid, 256, 0, st>>>(v, Q, kin);          \
    else score_mfma_kernel<BF, NBLK, true, false><<<grid, 256, 0, st>>>(v, Q, nullptr);         \
  } while (0)
    grid = score_grid(v);
    const bool two = v.G + (kin ? 1 : 0) > 16;
    if (v.dtype == DYNAKV_BF16) { if (two) DYNAKV_SCORE_B(true, 2); else DYNAKV_SCORE_B(true, 1); }
    else { if (two) DYNAKV_SCORE_B(false, 2); else DYNAKV_SCORE_B(false, 1); }
#undef DYNAKV_SCORE_B
  }
  if (v.Mcap > kSelectLds) select_kernel<true><<<v.U, 1024, 0, st>>>(v, Q, budget);
  else select_kernel<false><<<v.U, 1024, 0, st>>>(v, Q, budget);
  return hipGetLastError();
}

// The distances of a new key alone (an append outside a whole-step call, 16-bit search copy).
hipError_t launch_near(const View& v, const void* kin, hipStream_t st) {
  const dim3 grid = score_grid(v);
  if (v.dtype == DYNAKV_BF16) score_mfma_kernel<true, 1, false, true><<<grid, 256, 0, st>>>(v, nullptr, kin);
  else score_mfma_kernel<false, 1, false, true><<<grid, 256, 0, st>>>(v, nullptr, kin);
  return hipGetLastError();
}

hipError_t launch_gather_attend(const View& v, const void* Q, float* out, float* lse, hipStream_t st) {
  if (v.dtype == DYNAKV_F32) launch_ga<DYNAKV_F32, 4, true>(v, Q, out, lse, st);
  else if (v.dtype == DYNAKV_F16) launch_ga_dt<DYNAKV_F16>(v, Q, out, lse, st);
  else launch_ga_dt<DYNAKV_BF16>(v, Q, out, lse, st);
  return hipGetLastError();
}

}  // namespace dynakv
