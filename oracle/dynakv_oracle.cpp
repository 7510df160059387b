// CPU ORACLE for cluster-indexed sparse attention with adaptive cluster management.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, step-by-step
// implementation of the method of the DynaKV paper (Section 4.1, Eq. 1-5; Section 4.2;
// Algorithm 1; the k-means and attention remarks of Section 7), written to be checked
// against the paper by eye.  Only tests, the smoke check and the CPU-baseline leg of the
// benchmark may call it.  It shares no code with the GPU library.
//
// Arithmetic (the plain definitions, nothing blocked or reordered):
//   * inputs are float32 values (already rounded to the K/V storage type by the caller);
//   * every dot product, squared distance, sum, mean and variance is a float64 sum taken left
//     to right over the coordinate index 0..d-1; sums over members run in storage order;
//   * centroids are STORED as float32 (rounded once per update); M2 (= n * variance) and the
//     split threshold tau are stored as float64; ties go to the lowest index;
//   * two readings that the paper leaves open are configuration fields: which copy of a
//     centroid the searches read (`search_copy`: the mean rounded to the storage type of the
//     keys, or the float32 mean itself) and whether cluster scores are rounded to float32
//     before they are ordered (`score_round`).
// Every decision (nearest cluster, threshold test, budget cut, 2-means seeds and sides) also
// reports its normalised margin, so that a caller comparing another implementation against
// this one can tell a genuine disagreement from a tie below 1e-4.
//
// Pins: tests/test_oracle_pins.py (dense attention at budget >= N, scipy / scikit-learn special
// cases, closed forms, invariants, brute force on tiny inputs, hand-computed fixtures in
// tests/golden/).  Long trajectories at the real configuration sizes are pinned only
// through those per-step properties: "parity unpinned" beyond them.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

struct Config {
  int32_t n_units;          // independent (layer, sequence, KV head) units
  int32_t group_size;       // query heads per KV head (G)
  int32_t head_dim;         // d
  int32_t n_clusters_init;  // M0
  int32_t max_clusters;     // capacity, splits included
  int32_t max_tokens;       // capacity per unit
  int32_t kmeans_iters;     // Lloyd iterations, no early exit
  int32_t buffer_max;       // B_max of Algorithm 1 (0: every cluster counts as resident)
  int32_t group_reduce;     // 0: max over the group's heads, 1: sum
  float var_alpha;          // tau = var_alpha * (k-means objective / N0); <= 0: off
  float size_factor;        // split when n' > size_factor * mean cluster size; <= 0: off
  float softmax_scale;      // 0: 1/sqrt(d)
  int32_t dtype;            // storage type of K, V, Q: 0 float32, 1 float16, 2 bfloat16
  int32_t search_copy;      // 0: searches read r_j rounded to the storage type; 1: the float32 mean
  int32_t score_round;      // 0: clusters are ordered by their float64 scores; 1: rounded to float32 first
  int32_t update_mode;      // 0: Algorithm 1 (adaptive); 1: static update (entries join the nearest cluster,
                            //    statistics are updated, nothing is ever flagged or split: Section 2.3);
                            //    2: no clustering (the naive baseline of Section 8.1): every entry is a cluster of
                            //    its own, so retrieval is exact top-B over tokens;
                            //    3: local update (Section 2.3): new entries are clustered among themselves, apart from
                            //    the existing clusters: each becomes a cluster of its own until local_window of them
                            //    have come in, which a k-means of their own then turns into local_clusters clusters
  int32_t local_window;     // W (update_mode 3)
  int32_t local_clusters;   // k <= W (update_mode 3)
};

struct Cluster {
  int32_t n = 0;            // committed size n_j
  int32_t b = 0;            // |Buf_j|: the last b members are the buffered ones
  int32_t flag = 0;         // f_j = SPLIT
  double M2 = 0.0;          // n_j * sigma_j^2 of the committed members
  std::vector<float> r;     // centroid r_j, float32
  std::vector<float> rs;    // the copy of r_j that searches read (see search_copy)
  std::vector<int32_t> members;  // token positions in storage order
};

// Normalised margins of the decisions of the last call of each kind (infinity: no such decision was taken).
struct Margins {
  double assign = 0, trigger = 0, select = 0, split = 0;
};

struct Unit {
  int32_t N = 0;
  std::vector<float> K, V;          // [N][d] by token position
  std::vector<Cluster> clusters;
  double tau = 0.0;
  std::vector<int32_t> selected;    // ids in score order (P_req of the last retrieval)
  std::vector<uint8_t> in_req;      // bitmap of P_req by cluster id
  std::vector<int32_t> gather;      // token positions attended by the last retrieval
  std::vector<double> scores;       // last cluster scores (after score_round, if set)
  std::vector<double> kmeans_margin;  // per prefill point: smallest assignment margin over the Lloyd iterations
  int32_t last_assign = -1;
  int32_t local_count = 0;          // update_mode 3: entries since the last local clustering
  int32_t last_split_rounds = 0;    // Lloyd rounds of the most recent 2-means
  int32_t error = 0;
  int64_t n_splits = 0, n_failed_splits = 0, n_forced = 0;
  int64_t ties[5] = {0, 0, 0, 0, 0};   // kmeans, assign, trigger, select, split-side
  Margins mg;
};

struct Oracle {
  Config cfg;
  std::vector<Unit> units;
  int threads = 0;
};

constexpr double kTieMargin = 1e-4;
constexpr double kInf = std::numeric_limits<double>::infinity();

// ---- the arithmetic primitives everything else is made of ---------------------------------

// float64 dot product of two float32 vectors, left to right.
inline double dot_ff(const float* a, const float* b, int d) {
  double acc = 0.0;
  for (int i = 0; i < d; ++i) acc += (double)a[i] * (double)b[i];
  return acc;
}
// float64 squared distance between a float32 point and a float32 centre.
inline double sqdist_ff(const float* x, const float* c, int d) {
  double acc = 0.0;
  for (int i = 0; i < d; ++i) {
    const double t = (double)x[i] - (double)c[i];
    acc += t * t;
  }
  return acc;
}
// Same, centre held in float64 (used inside a split, where centres are not rounded).
inline double sqdist_fd(const float* x, const double* c, int d) {
  double acc = 0.0;
  for (int i = 0; i < d; ++i) {
    const double t = (double)x[i] - c[i];
    acc += t * t;
  }
  return acc;
}

// Round to nearest, ties to even, onto the grid of a binary format with `mant` explicit mantissa bits, smallest
// normal exponent `emin` and largest finite value `fmax` (IEEE-style: gradual underflow, overflow to infinity).
inline float round_to_format(float x, int mant, int emin, double fmax) {
  if (x == 0.f || !std::isfinite(x)) return x;
  int e;
  std::frexp((double)x, &e);                        // |x| = f * 2^e with f in [0.5, 1): floor(log2|x|) = e - 1
  const int ex = std::max(e - 1, emin);
  const double quantum = std::ldexp(1.0, ex - mant);
  const double y = std::nearbyint((double)x / quantum) * quantum;   // default rounding mode: ties to even
  if (std::fabs(y) > fmax) return (float)std::copysign(kInf, y);
  return (float)y;
}
inline float round_to_storage(float x, int dtype) {
  if (dtype == 1) return round_to_format(x, 10, -14, 65504.0);                                   // float16
  if (dtype == 2) return round_to_format(x, 7, -126, std::ldexp(2.0 - std::ldexp(1.0, -7), 127));   // bfloat16
  return x;
}

// Margin of a decision between two candidate values a (taken) and b (runner-up): their gap over the larger of
// 1, |a| and |b|.
inline double norm_margin(double gap, double a, double b) {
  return gap / std::max(1.0, std::max(std::fabs(a), std::fabs(b)));
}

// The representatives that a search reads (query similarity, Section 4.1; nearest cluster of a new entry,
// Algorithm 1).  The paper fixes no precision for them.  search_copy = 0: kept in the storage type of the keys,
// like the entries they stand for; 1: the float32 mean itself.  The statistics (float32 mean, M2) are not
// touched by this.  Called whenever r_j changes.
void search_copy(const Config& c, Cluster& cl) {
  cl.rs.resize(cl.r.size());
  for (size_t i = 0; i < cl.r.size(); ++i) cl.rs[i] = c.search_copy == 0 ? round_to_storage(cl.r[i], c.dtype) : cl.r[i];
}

// Nearest centre of x among all clusters (Algorithm 1, "assign to nearest cluster";
// squared Euclidean distance, the k-means metric).  Ties -> lowest id.
int nearest_cluster(const Unit& u, const float* x, int d, double* best_out, double* second_out) {
  double best = kInf, second = kInf;
  int arg = -1;
  for (int j = 0; j < (int)u.clusters.size(); ++j) {
    const double dj = sqdist_ff(x, u.clusters[j].rs.data(), d);
    if (dj < best) { second = best; best = dj; arg = j; }
    else if (dj < second) second = dj;
  }
  if (best_out) *best_out = best;
  if (second_out) *second_out = second;
  return arg;
}

// Exact two-pass statistics of a member list: n, float32 mean (Eq. 4), M2 about that mean.
void exact_stats(const Unit& u, const std::vector<int32_t>& mem, int d, std::vector<float>& r, double& M2) {
  std::vector<double> s(d, 0.0);
  for (int32_t p : mem)
    for (int i = 0; i < d; ++i) s[i] += (double)u.K[(size_t)p * d + i];
  r.assign(d, 0.f);
  if (!mem.empty())
    for (int i = 0; i < d; ++i) r[i] = (float)(s[i] / (double)mem.size());
  M2 = 0.0;
  for (int32_t p : mem) M2 += sqdist_ff(&u.K[(size_t)p * d], r.data(), d);
}

// ---- prefill: NewCluster(K0) = Lloyd's k-means (Section 4.1, Eq. 3-4; Algorithm 1) ----

int build_unit(const Config& c, Unit& u, const float* K, const float* V, int N0, const int32_t* init_idx,
               double* J_hist) {
  const int d = c.head_dim, M0 = c.n_clusters_init, T = c.kmeans_iters;
  u = Unit();
  u.N = N0;
  u.K.assign(K, K + (size_t)N0 * d);
  u.V.assign(V, V + (size_t)N0 * d);

  // initial centres: the M0 distinct points the caller names
  std::vector<float> R((size_t)M0 * d);
  for (int j = 0; j < M0; ++j) {
    const int32_t p = init_idx[j];
    if (p < 0 || p >= N0) return 1;
    std::copy(&u.K[(size_t)p * d], &u.K[(size_t)p * d] + d, &R[(size_t)j * d]);
  }

  std::vector<int32_t> label(N0, 0), count(M0, 0);
  std::vector<double> dist(N0, 0.0);
  u.kmeans_margin.assign(N0, kInf);
  for (int it = 0; it < T; ++it) {
    // (a) assignment: nearest centre, ties -> lowest j
    double J = 0.0;
    for (int i = 0; i < N0; ++i) {
      const float* x = &u.K[(size_t)i * d];
      double best = kInf, second = kInf;
      int arg = 0;
      for (int j = 0; j < M0; ++j) {
        const double dj = sqdist_ff(x, &R[(size_t)j * d], d);
        if (dj < best) { second = best; best = dj; arg = j; }
        else if (dj < second) second = dj;
      }
      label[i] = arg;
      dist[i] = best;
      J += best;
      if (M0 > 1) {
        const double xx = dot_ff(x, x, d);
        u.kmeans_margin[i] = std::min(u.kmeans_margin[i], norm_margin(second - best, xx - best, xx - second));
      }
    }
    if (J_hist) J_hist[it] = J;
    // (b) update: centre = mean of members (Eq. 4), float64 sum in position order, float32 store
    std::fill(count.begin(), count.end(), 0);
    std::vector<double> S((size_t)M0 * d, 0.0);
    for (int i = 0; i < N0; ++i) {
      ++count[label[i]];
      double* s = &S[(size_t)label[i] * d];
      const float* x = &u.K[(size_t)i * d];
      for (int k = 0; k < d; ++k) s[k] += (double)x[k];
    }
    for (int j = 0; j < M0; ++j)
      if (count[j] > 0)
        for (int k = 0; k < d; ++k) R[(size_t)j * d + k] = (float)(S[(size_t)j * d + k] / (double)count[j]);
    // (c) empty clusters (all iterations but the last): in ascending id, each takes the
    //     not-yet-taken point that is farthest from its own centre (ties -> lowest i).
    if (it + 1 < T) {
      std::vector<uint8_t> taken(N0, 0);
      for (int j = 0; j < M0; ++j) {
        if (count[j] > 0) continue;
        int far = -1;
        for (int i = 0; i < N0; ++i)
          if (!taken[i] && (far < 0 || dist[i] > dist[far])) far = i;
        if (far < 0) break;
        taken[far] = 1;
        std::copy(&u.K[(size_t)far * d], &u.K[(size_t)far * d] + d, &R[(size_t)j * d]);
      }
    }
  }
  for (int i = 0; i < N0; ++i) u.ties[0] += u.kmeans_margin[i] <= kTieMargin;

  // cluster records: members in ascending position, n, r, M2 about the stored centre
  u.clusters.assign(M0, Cluster());
  for (int j = 0; j < M0; ++j) u.clusters[j].r.assign(&R[(size_t)j * d], &R[(size_t)j * d] + d);
  for (int i = 0; i < N0; ++i) u.clusters[label[i]].members.push_back(i);
  double Jfinal = 0.0;
  for (int j = 0; j < M0; ++j) {
    Cluster& cl = u.clusters[j];
    cl.n = (int32_t)cl.members.size();
    cl.M2 = 0.0;
    for (int32_t p : cl.members) cl.M2 += sqdist_ff(&u.K[(size_t)p * d], cl.r.data(), d);
    Jfinal += cl.M2;
    search_copy(c, cl);
  }
  // head-specific threshold: a multiple of the unit's own mean squared distance to centre
  u.tau = (double)c.var_alpha * (Jfinal / (double)N0);
  u.in_req.assign(M0, 0);
  u.mg = Margins{kInf, kInf, kInf, kInf};
  return 0;
}

// ---- decode: retrieval + attention over the retrieved set (Section 4.1; Algorithm 1) ----

void retrieve_attend_unit(const Config& c, Unit& u, const float* Q, int budget, double* out, double* lse) {
  const int d = c.head_dim, G = c.group_size, M = (int)u.clusters.size();
  const double scale = c.softmax_scale > 0.f ? (double)c.softmax_scale : 1.0 / std::sqrt((double)d);

  // query-representative similarity: inner product per head, reduced over the group
  u.scores.assign(M, 0.0);
  for (int j = 0; j < M; ++j) {
    double red = 0.0;
    for (int g = 0; g < G; ++g) {
      const double s = dot_ff(Q + (size_t)g * d, u.clusters[j].rs.data(), d);
      if (g == 0) red = s;
      else if (c.group_reduce == 0) red = std::max(red, s);
      else red += s;
    }
    u.scores[j] = c.score_round ? (double)(float)(red * scale) : red * scale;
  }
  // order by (score desc, id asc)
  std::vector<int32_t> order(M);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return u.scores[a] > u.scores[b]; });

  // top-k under the token budget: longest prefix whose stored sizes fit
  u.selected.clear();
  u.gather.clear();
  u.in_req.assign(M, 0);
  int64_t used = 0;
  int cut = 0;
  for (; cut < M; ++cut) {
    const Cluster& cl = u.clusters[order[cut]];
    const int64_t sz = (int64_t)cl.members.size();
    if (used + sz > budget) break;
    used += sz;
  }
  if (cut == 0 && M > 0 && budget > 0) {  // the best cluster alone is over budget: its first `budget` members
    const Cluster& cl = u.clusters[order[0]];
    u.selected.push_back(order[0]);
    u.in_req[order[0]] = 1;
    for (int i = 0; i < budget; ++i) u.gather.push_back(cl.members[i]);
  } else {
    for (int r = 0; r < cut; ++r) {
      const Cluster& cl = u.clusters[order[r]];
      u.selected.push_back(order[r]);
      u.in_req[order[r]] = 1;
      for (int32_t p : cl.members) u.gather.push_back(p);
    }
  }
  // selection margin: the two score gaps around the cut (last taken vs first left out, first left out vs next)
  u.mg.select = kInf;
  for (int r = cut; r <= cut + 1; ++r)
    if (r >= 1 && r < M) {
      const double a = u.scores[order[r - 1]], b = u.scores[order[r]];
      u.mg.select = std::min(u.mg.select, norm_margin(a - b, a, b));
    }
  if (u.mg.select <= kTieMargin) ++u.ties[3];

  // softmax attention over the gathered entries, any order (max-subtracted)
  for (int g = 0; g < G; ++g) {
    const float* q = Q + (size_t)g * d;
    const size_t T = u.gather.size();
    std::vector<double> logit(T);
    double mx = -kInf;
    for (size_t t = 0; t < T; ++t) {
      logit[t] = scale * dot_ff(q, &u.K[(size_t)u.gather[t] * d], d);
      mx = std::max(mx, logit[t]);
    }
    double den = 0.0;
    std::vector<double> acc(d, 0.0);
    for (size_t t = 0; t < T; ++t) {
      const double p = std::exp(logit[t] - mx);
      den += p;
      const float* v = &u.V[(size_t)u.gather[t] * d];
      for (int k = 0; k < d; ++k) acc[k] += p * (double)v[k];
    }
    for (int k = 0; k < d; ++k) out[(size_t)g * d + k] = T ? acc[k] / den : 0.0;
    if (lse) lse[g] = T ? mx + std::log(den) : -kInf;
  }
}

// ---- local update (Section 2.3): the last W entries, each a cluster of its own so far, are clustered among
// themselves by Lloyd's k-means into k clusters that take their place (ids M - W .. M - W + k - 1).  Initial centres:
// the entries 0, W/k, 2W/k, ... of the window (integer division); kmeans_iters iterations of assign (nearest
// centre, ties to the lowest) and update (mean of the members, stored as float32; a centre without members stays
// where it is); members in ascending position; exact statistics about the stored centre.
void local_recluster(const Config& c, Unit& u) {
  const int d = c.head_dim, W = c.local_window, k = c.local_clusters;
  const int base = (int)u.clusters.size() - W;
  std::vector<int32_t> pos(W);
  for (int i = 0; i < W; ++i) pos[i] = u.clusters[base + i].members[0];
  auto X = [&](int i) { return &u.K[(size_t)pos[i] * d]; };
  std::vector<float> R((size_t)k * d);
  for (int j = 0; j < k; ++j) std::copy(X(j * W / k), X(j * W / k) + d, &R[(size_t)j * d]);
  std::vector<int32_t> label(W, 0);
  for (int it = 0; it < c.kmeans_iters; ++it) {
    for (int i = 0; i < W; ++i) {
      double best = kInf, second = kInf;
      int arg = 0;
      for (int j = 0; j < k; ++j) {
        const double dj = sqdist_ff(X(i), &R[(size_t)j * d], d);
        if (dj < best) { second = best; best = dj; arg = j; }
        else if (dj < second) second = dj;
      }
      label[i] = arg;
      if (k > 1) {
        const double xx = dot_ff(X(i), X(i), d);
        u.mg.split = std::min(u.mg.split, norm_margin(second - best, xx - best, xx - second));
      }
    }
    std::vector<double> S((size_t)k * d, 0.0);
    std::vector<int32_t> cnt(k, 0);
    for (int i = 0; i < W; ++i) {
      ++cnt[label[i]];
      for (int t = 0; t < d; ++t) S[(size_t)label[i] * d + t] += (double)X(i)[t];
    }
    for (int j = 0; j < k; ++j)
      if (cnt[j] > 0)
        for (int t = 0; t < d; ++t) R[(size_t)j * d + t] = (float)(S[(size_t)j * d + t] / (double)cnt[j]);
  }
  std::vector<Cluster> fresh(k);
  for (int j = 0; j < k; ++j) fresh[j].r.assign(&R[(size_t)j * d], &R[(size_t)j * d] + d);
  for (int i = 0; i < W; ++i) fresh[label[i]].members.push_back(pos[i]);
  for (int j = 0; j < k; ++j) {
    Cluster& cl = fresh[j];
    cl.n = (int32_t)cl.members.size();
    cl.M2 = 0.0;
    for (int32_t p : cl.members) cl.M2 += sqdist_ff(&u.K[(size_t)p * d], cl.r.data(), d);
    search_copy(c, cl);
  }
  u.clusters.resize(base);
  for (int j = 0; j < k; ++j) u.clusters.push_back(fresh[j]);
  u.in_req.assign(u.clusters.size(), 0);
  if (u.mg.split <= kTieMargin) ++u.ties[4];
}

// ---- decode: assign + UpdateVar + keep / flag (Algorithm 1; Section 4.2) ----------------

void append_unit(const Config& c, Unit& u, const float* k, const float* v) {
  const int d = c.head_dim, M = (int)u.clusters.size();
  if (u.N >= c.max_tokens || M == 0) { u.error |= 1; return; }
  if (c.update_mode == 2 || c.update_mode == 3) {   // the entry becomes cluster M, its own representative
    if (M >= c.max_clusters) { u.error |= 2; return; }
    Cluster cl;
    cl.n = 1;
    cl.r.assign(k, k + d);
    cl.members.push_back(u.N);
    search_copy(c, cl);
    u.K.insert(u.K.end(), k, k + d);
    u.V.insert(u.V.end(), v, v + d);
    u.N += 1;
    u.clusters.push_back(cl);
    u.in_req.push_back(0);
    u.last_assign = M;
    u.mg.assign = kInf; u.mg.trigger = kInf; u.mg.split = kInf;
    if (c.update_mode == 3 && ++u.local_count == c.local_window) {
      local_recluster(c, u);
      u.local_count = 0;
    }
    return;
  }
  double best, second;
  const int j = nearest_cluster(u, k, d, &best, &second);
  u.last_assign = j;
  {
    const double xx = dot_ff(k, k, d);
    u.mg.assign = M > 1 ? norm_margin(second - best, xx - best, xx - second) : kInf;
    if (u.mg.assign <= kTieMargin) ++u.ties[1];
  }
  const int32_t pos = u.N;
  u.K.insert(u.K.end(), k, k + d);
  u.V.insert(u.V.end(), v, v + d);
  u.N += 1;
  Cluster& cl = u.clusters[j];
  cl.members.push_back(pos);          // stored with its cluster whatever the branch
  u.mg.trigger = kInf;
  if (cl.flag) { cl.b += 1; return; }  // already flagged: goes to Buf_j

  // UpdateVar: tentative size, centroid and M2 from (n, r, M2) and the new entry alone
  const int32_t n1 = cl.n + 1;
  std::vector<double> r1(d);
  for (int i = 0; i < d; ++i) r1[i] = (double)cl.r[i] + ((double)k[i] - (double)cl.r[i]) / (double)n1;
  double M2 = cl.M2;
  for (int i = 0; i < d; ++i) M2 += ((double)k[i] - (double)cl.r[i]) * ((double)k[i] - r1[i]);   // delta_i * (k_i - r'_i)
  const double var1 = M2 / (double)n1;
  bool trig = false;
  if (n1 >= 2 && c.update_mode == 0) {
    if (c.var_alpha > 0.f) {
      if (var1 > u.tau) trig = true;
      u.mg.trigger = std::fabs(var1 - u.tau) / std::max(1.0, u.tau);
      if (u.mg.trigger <= kTieMargin) ++u.ties[2];
    }
    // size trigger: n' > size_factor * (N_t + 1) / M_t, N_t counted before this append
    if (c.size_factor > 0.f && (double)n1 * (double)M > (double)c.size_factor * (double)(pos + 1)) trig = true;
  }
  if (!trig) {                        // AddEntry + UpdateStats
    cl.n = n1;
    for (int i = 0; i < d; ++i) cl.r[i] = (float)r1[i];
    cl.M2 = M2;
    search_copy(c, cl);
  } else {                            // statistics stay frozen; entry buffered, cluster flagged
    cl.flag = 1;
    cl.b = 1;
  }
}

// ---- SplitCluster: local 2-means on one cluster (Algorithm 1; Sections 4.2, 5.2) --------

// Gap between the largest and the second largest of v (ties: 0), over the larger of 1 and the largest.
double top_gap(const std::vector<double>& v) {
  double a = -kInf, b = -kInf;
  for (double t : v) {
    if (t > a) { b = a; a = t; }
    else if (t > b) b = t;
  }
  return v.size() < 2 ? kInf : (a - b) / std::max(1.0, a);
}

// Returns 1 if split, 0 if it could not be split (flag cleared, statistics made exact),
// -1 if there is no room for a new cluster (left flagged).
int split_cluster(const Config& c, Unit& u, int j) {
  const int d = c.head_dim;
  Cluster& cl = u.clusters[j];
  const std::vector<int32_t> mem = cl.members;
  const int m = (int)mem.size();
  u.last_split_rounds = 0;
  auto fail = [&]() {
    exact_stats(u, cl.members, d, cl.r, cl.M2);
    search_copy(c, cl);
    cl.n = m; cl.b = 0; cl.flag = 0;
    ++u.n_failed_splits;
    return 0;
  };
  if (m < 2) return fail();
  auto X = [&](int i) { return &u.K[(size_t)mem[i] * d]; };

  // seeds: A = farthest from the mean of all members, B = farthest from A (ties -> earliest)
  std::vector<double> mean(d, 0.0);
  for (int i = 0; i < m; ++i)
    for (int k = 0; k < d; ++k) mean[k] += (double)X(i)[k];
  for (int k = 0; k < d; ++k) mean[k] /= (double)m;
  std::vector<double> dm(m), da(m);
  int a = 0;
  for (int i = 0; i < m; ++i) { dm[i] = sqdist_fd(X(i), mean.data(), d); if (dm[i] > dm[a]) a = i; }
  int b = 0;
  for (int i = 0; i < m; ++i) { da[i] = sqdist_ff(X(i), X(a), d); if (da[i] > da[b]) b = i; }
  if (!(da[b] > 0.0)) return fail();     // all members identical
  u.mg.split = std::min(u.mg.split, std::min(top_gap(dm), top_gap(da)));

  std::vector<double> cA(d), cB(d);
  for (int k = 0; k < d; ++k) { cA[k] = (double)X(a)[k]; cB[k] = (double)X(b)[k]; }
  std::vector<uint8_t> side(m, 2), nside(m);
  for (int it = 0; it < 16; ++it) {
    for (int i = 0; i < m; ++i) {
      const double dA = sqdist_fd(X(i), cA.data(), d), dB = sqdist_fd(X(i), cB.data(), d);
      nside[i] = dA <= dB ? 0 : 1;    // tie -> side A
      const double xx = dot_ff(X(i), X(i), d);
      const double mg = norm_margin(std::fabs(dA - dB), xx - dA, xx - dB);
      u.mg.split = std::min(u.mg.split, mg);
      if ((it == 0 || nside[i] != side[i]) && mg <= kTieMargin) ++u.ties[4];
    }
    if (nside == side) break;
    side = nside;
    u.last_split_rounds = it + 1;
    int nA = 0;
    for (int i = 0; i < m; ++i) nA += side[i] == 0;
    if (nA == 0 || nA == m) return fail();
    std::vector<double> sA(d, 0.0), sB(d, 0.0);
    for (int i = 0; i < m; ++i) {
      double* s = side[i] == 0 ? sA.data() : sB.data();
      for (int k = 0; k < d; ++k) s[k] += (double)X(i)[k];
    }
    for (int k = 0; k < d; ++k) { cA[k] = sA[k] / (double)nA; cB[k] = sB[k] / (double)(m - nA); }
  }
  if ((int)u.clusters.size() >= c.max_clusters) { u.error |= 2; return -1; }

  // children keep storage order; the one holding the earliest entry keeps id j
  const uint8_t keep = side[0];
  Cluster stay, moved;
  for (int i = 0; i < m; ++i) (side[i] == keep ? stay : moved).members.push_back(mem[i]);
  for (Cluster* ch : {&stay, &moved}) {
    exact_stats(u, ch->members, d, ch->r, ch->M2);
    search_copy(c, *ch);
    ch->n = (int32_t)ch->members.size();
    ch->b = 0; ch->flag = 0;
  }
  u.clusters[j] = stay;
  u.clusters.push_back(moved);
  u.in_req.push_back(0);              // a new cluster is not part of this step's active set
  ++u.n_splits;
  return 1;
}

void split_unit(const Config& c, Unit& u) {
  if (c.update_mode != 0) return;     // nothing is ever flagged (and a local clustering has left its margin)
  u.mg.split = kInf;
  // delayed splits: flagged clusters that the last retrieval brought in
  const int M = (int)u.clusters.size();
  for (int j = 0; j < M; ++j) {
    const Cluster& cl = u.clusters[j];
    if (cl.flag && (c.buffer_max == 0 || (j < (int)u.in_req.size() && u.in_req[j]))) split_cluster(c, u, j);
  }
  // forced split once the buffers hold B_max entries: the cluster with the fullest buffer (lowest id among equals)
  if (c.buffer_max > 0) {
    int64_t tot = 0; int arg = -1;
    for (int j = 0; j < (int)u.clusters.size(); ++j) {
      const Cluster& cl = u.clusters[j];
      if (!cl.flag) continue;
      tot += cl.b;
      if (arg < 0 || cl.b > u.clusters[arg].b) arg = j;
    }
    if (arg >= 0 && tot >= c.buffer_max) {
      if (split_cluster(c, u, arg) == 1) ++u.n_forced;    // counted when the split was carried out
    }
  }
}

}  // namespace

// ---- C interface (ctypes) ------------------------------------------------------------------

extern "C" {

struct oracle_config {
  int32_t n_units, group_size, head_dim, n_clusters_init, max_clusters, max_tokens, kmeans_iters, buffer_max,
      group_reduce;
  float var_alpha, size_factor, softmax_scale;
  int32_t dtype, search_copy, score_round, update_mode, local_window, local_clusters;
};

void* oracle_create(const oracle_config* c) {
  Oracle* o = new Oracle();
  o->cfg = Config{c->n_units, c->group_size, c->head_dim, c->n_clusters_init, c->max_clusters, c->max_tokens,
                  c->kmeans_iters, c->buffer_max, c->group_reduce, c->var_alpha, c->size_factor, c->softmax_scale,
                  c->dtype, c->search_copy, c->score_round, c->update_mode, c->local_window, c->local_clusters};
  o->units.resize(c->n_units);
  return o;
}
void oracle_destroy(void* h) { delete (Oracle*)h; }
void oracle_set_threads(void* h, int t) { ((Oracle*)h)->threads = t; }
int oracle_threads_used(void* h) {
  Oracle* o = (Oracle*)h;
#ifdef _OPENMP
  const int t = o->threads > 0 ? o->threads : omp_get_max_threads();
  return std::min(t, (int)o->units.size());
#else
  (void)o; return 1;
#endif
}

#ifdef _OPENMP
#define UNIT_LOOP(o) \
  _Pragma("omp parallel for schedule(dynamic, 1) num_threads(oracle_threads_used(o))")
#else
#define UNIT_LOOP(o)
#endif

// K, V: [U][n_tokens][d] float32; init_idx: [U][M0], positions of the initial centres; J_hist: [U][iters] or null.
int oracle_build_index(void* h, const float* K, const float* V, int n_tokens, const int32_t* init_idx,
                       double* J_hist) {
  Oracle* o = (Oracle*)h;
  const Config& c = o->cfg;
  if (!init_idx || n_tokens < c.n_clusters_init || n_tokens > c.max_tokens || c.n_clusters_init > c.max_clusters ||
      c.n_clusters_init < 1 || c.kmeans_iters < 1)
    return 1;
  const size_t stride = (size_t)n_tokens * c.head_dim;
  std::vector<int> rc(c.n_units, 0);
  UNIT_LOOP(o)
  for (int u = 0; u < c.n_units; ++u)
    rc[u] = build_unit(c, o->units[u], K + u * stride, V + u * stride, n_tokens, init_idx + (size_t)u * c.n_clusters_init,
                       J_hist ? J_hist + (size_t)u * c.kmeans_iters : nullptr);
  for (int r : rc)
    if (r) return 1;
  return 0;
}

// Replaces the state of unit u by the given one (the counterpart of the GPU library's exported state):
// K, V [N][d] float32 by token position; per cluster centroids [M][d] float32, n, b, flag [M], M2 [M] float64;
// offsets [M+1] and members [N]: token positions of cluster j in storage order = members[offsets[j]..offsets[j+1]);
// selected [n_sel]: ids of the last active set.  Returns nonzero on inconsistent sizes.
int oracle_import_unit(void* h, int u, int N, const float* K, const float* V, int M, const float* centroids,
                       const int32_t* n, const int32_t* b, const int32_t* flag, const double* M2,
                       const int32_t* offsets, const int32_t* members, double tau, int n_sel, const int32_t* selected) {
  Oracle* o = (Oracle*)h;
  const Config& c = o->cfg;
  const int d = c.head_dim;
  if (u < 0 || u >= c.n_units || N < 0 || N > c.max_tokens || M < 1 || M > c.max_clusters || offsets[M] != N) return 1;
  Unit nu;
  nu.N = N;
  nu.K.assign(K, K + (size_t)N * d);
  nu.V.assign(V, V + (size_t)N * d);
  nu.clusters.assign(M, Cluster());
  for (int j = 0; j < M; ++j) {
    Cluster& cl = nu.clusters[j];
    cl.n = n[j]; cl.b = b[j]; cl.flag = flag[j]; cl.M2 = M2[j];
    if (offsets[j + 1] - offsets[j] != n[j] + b[j]) return 1;
    cl.r.assign(centroids + (size_t)j * d, centroids + (size_t)(j + 1) * d);
    cl.members.assign(members + offsets[j], members + offsets[j + 1]);
    search_copy(c, cl);
  }
  nu.tau = tau;
  nu.in_req.assign(M, 0);
  for (int i = 0; i < n_sel; ++i) {
    if (selected[i] < 0 || selected[i] >= M) return 1;
    nu.selected.push_back(selected[i]);
    nu.in_req[selected[i]] = 1;
  }
  nu.mg = Margins{kInf, kInf, kInf, kInf};
  // counters carry over: they describe the run, not the state
  const Unit& old = o->units[u];
  nu.n_splits = old.n_splits; nu.n_failed_splits = old.n_failed_splits; nu.n_forced = old.n_forced;
  std::copy(old.ties, old.ties + 5, nu.ties);
  nu.last_assign = old.last_assign;
  nu.error = old.error;
  nu.local_count = old.local_count;
  o->units[u] = std::move(nu);
  return 0;
}

// Q: [U][G][d]; out: [U][G][d] float64; lse: [U][G] float64 or null.
int oracle_retrieve_attend(void* h, const float* Q, int budget, double* out, double* lse) {
  Oracle* o = (Oracle*)h;
  const Config& c = o->cfg;
  const size_t qs = (size_t)c.group_size * c.head_dim;
  UNIT_LOOP(o)
  for (int u = 0; u < c.n_units; ++u)
    retrieve_attend_unit(c, o->units[u], Q + u * qs, budget, out + u * qs, lse ? lse + (size_t)u * c.group_size : nullptr);
  return 0;
}

// k, v: [U][d]
int oracle_append(void* h, const float* k, const float* v) {
  Oracle* o = (Oracle*)h;
  const Config& c = o->cfg;
  UNIT_LOOP(o)
  for (int u = 0; u < c.n_units; ++u)
    append_unit(c, o->units[u], k + (size_t)u * c.head_dim, v + (size_t)u * c.head_dim);
  return 0;
}

// Adaptive clustering applied continuously through a long prefill (Section 7, Discussion 1): n more entries per
// unit, one after the other, each assigned, tested against the threshold and, since the chunk is resident, split
// at once where flagged (the decode block of Algorithm 1 with every cluster in memory).  K, V: [U][n][d].
int oracle_extend(void* h, const float* K, const float* V, int n) {
  Oracle* o = (Oracle*)h;
  Config c = o->cfg;
  c.buffer_max = 0;
  const size_t stride = (size_t)n * c.head_dim;
  UNIT_LOOP(o)
  for (int u = 0; u < c.n_units; ++u)
    for (int t = 0; t < n; ++t) {
      append_unit(c, o->units[u], K + u * stride + (size_t)t * c.head_dim, V + u * stride + (size_t)t * c.head_dim);
      split_unit(c, o->units[u]);
    }
  return 0;
}

// Inter-cluster correlation (Section 5.1, Eq. 8).  n_ref reference retrievals (query similarity and budget cut as
// in a decode step; no attention) on the index as it stands; f(i, j) = number of them that select both cluster i and
// cluster j (i != j; the diagonal stays 0), P(i, j) = f(i, j) / sum over all ordered pairs.  The placement order
// puts highly correlated clusters next to each other: a greedy chain that starts at the cluster with the largest
// total co-retrieval count and always continues with the not yet placed cluster that is co-retrieved most often with
// the last one (lowest id among equals, also at the start).
// Q: [n_ref][U][G][d]; P: [U][M][M] float64 (or null); order: [U][M] (or null); M = clusters of unit 0 = of every unit.
int oracle_coretrieval(void* h, const float* Q, int n_ref, int budget, double* P, int32_t* order) {
  Oracle* o = (Oracle*)h;
  const Config& c = o->cfg;
  const size_t qs = (size_t)c.group_size * c.head_dim;
  const int M = (int)o->units[0].clusters.size();
  for (const Unit& un : o->units)
    if ((int)un.clusters.size() != M) return 1;
  UNIT_LOOP(o)
  for (int u = 0; u < c.n_units; ++u) {
    Unit& un = o->units[u];
    std::vector<int64_t> f((size_t)M * M, 0);
    std::vector<double> out(qs), lse(c.group_size);
    for (int r = 0; r < n_ref; ++r) {
      retrieve_attend_unit(c, un, Q + ((size_t)r * c.n_units + u) * qs, budget, out.data(), lse.data());
      for (int32_t a : un.selected)
        for (int32_t b : un.selected)
          if (a != b) ++f[(size_t)a * M + b];
    }
    int64_t total = 0;
    for (int64_t x : f) total += x;
    if (P)
      for (size_t i = 0; i < f.size(); ++i) P[(size_t)u * M * M + i] = total ? (double)f[i] / (double)total : 0.0;
    if (order) {
      std::vector<uint8_t> placed(M, 0);
      int last = 0;
      int64_t best = -1;
      for (int i = 0; i < M; ++i) {
        int64_t row = 0;
        for (int j = 0; j < M; ++j) row += f[(size_t)i * M + j];
        if (row > best) { best = row; last = i; }
      }
      for (int k = 0; k < M; ++k) {
        order[(size_t)u * M + k] = last;
        placed[last] = 1;
        int next = -1;
        for (int j = 0; j < M; ++j)
          if (!placed[j] && (next < 0 || f[(size_t)last * M + j] > f[(size_t)last * M + next])) next = j;
        last = next;
      }
    }
  }
  return 0;
}

int oracle_split(void* h) {
  Oracle* o = (Oracle*)h;
  UNIT_LOOP(o)
  for (int u = 0; u < o->cfg.n_units; ++u) split_unit(o->cfg, o->units[u]);
  return 0;
}

int oracle_num_clusters(void* h, int u) { return (int)((Oracle*)h)->units[u].clusters.size(); }
int oracle_num_tokens(void* h, int u) { return ((Oracle*)h)->units[u].N; }
int oracle_error(void* h, int u) { return ((Oracle*)h)->units[u].error; }
double oracle_tau(void* h, int u) { return ((Oracle*)h)->units[u].tau; }
int oracle_last_assign(void* h, int u) { return ((Oracle*)h)->units[u].last_assign; }
int oracle_last_split_rounds(void* h, int u) { return ((Oracle*)h)->units[u].last_split_rounds; }

// centroids [M][d] f32, n/b/flag [M] i32, M2 [M] f64 (any may be null)
void oracle_get_clusters(void* h, int u, float* centroids, int32_t* n, int32_t* b, int32_t* flag, double* M2) {
  const Oracle* o = (Oracle*)h;
  const Unit& un = o->units[u];
  const int d = o->cfg.head_dim;
  for (size_t j = 0; j < un.clusters.size(); ++j) {
    const Cluster& cl = un.clusters[j];
    if (centroids) std::copy(cl.r.begin(), cl.r.end(), centroids + j * d);
    if (n) n[j] = cl.n;
    if (b) b[j] = cl.b;
    if (flag) flag[j] = cl.flag;
    if (M2) M2[j] = cl.M2;
  }
}
// offsets [M+1], members [N] (positions in storage order, cluster after cluster)
void oracle_get_members(void* h, int u, int32_t* offsets, int32_t* members) {
  const Unit& un = ((Oracle*)h)->units[u];
  int32_t off = 0;
  for (size_t j = 0; j < un.clusters.size(); ++j) {
    offsets[j] = off;
    for (int32_t p : un.clusters[j].members) members[off++] = p;
  }
  offsets[un.clusters.size()] = off;
}
int oracle_get_selected(void* h, int u, int32_t* ids, int cap) {
  const Unit& un = ((Oracle*)h)->units[u];
  const int n = (int)un.selected.size();
  for (int i = 0; i < n && i < cap; ++i) ids[i] = un.selected[i];
  return n;
}
int oracle_get_gather(void* h, int u, int32_t* pos, int cap) {
  const Unit& un = ((Oracle*)h)->units[u];
  const int n = (int)un.gather.size();
  for (int i = 0; i < n && i < cap; ++i) pos[i] = un.gather[i];
  return n;
}
// keys and values by token position, [N][d] float32 each (either may be null)
void oracle_get_kv(void* h, int u, float* K, float* V) {
  const Unit& un = ((Oracle*)h)->units[u];
  if (K) std::copy(un.K.begin(), un.K.end(), K);
  if (V) std::copy(un.V.begin(), un.V.end(), V);
}
// the copies of the centroids that searches read, [M][d] f32
void oracle_get_search_copy(void* h, int u, float* out) {
  const Oracle* o = (Oracle*)h;
  const int d = o->cfg.head_dim;
  const Unit& un = o->units[u];
  for (size_t j = 0; j < un.clusters.size(); ++j) std::copy(un.clusters[j].rs.begin(), un.clusters[j].rs.end(), out + j * d);
}
// out[i] = in[i] rounded to the storage type (0 float32, 1 float16, 2 bfloat16), returned as float32
void oracle_round_to_storage(const float* in, float* out, int64_t n, int dtype) {
  for (int64_t i = 0; i < n; ++i) out[i] = round_to_storage(in[i], dtype);
}

void oracle_get_scores(void* h, int u, double* s) {
  const Unit& un = ((Oracle*)h)->units[u];
  std::copy(un.scores.begin(), un.scores.end(), s);
}
// per prefill point, the smallest margin of its nearest-centre decisions over the Lloyd iterations, [N0]
void oracle_get_kmeans_margins(void* h, int u, double* out) {
  const Unit& un = ((Oracle*)h)->units[u];
  std::copy(un.kmeans_margin.begin(), un.kmeans_margin.end(), out);
}
// margins[4] = assign, trigger, select, split (smallest over the last call's 2-means decisions) of the last
// calls; ties[5] = counts of decisions whose margin was <= 1e-4 (k-means points, assignments, triggers,
// selections, split sides); events[3] = splits, failed splits, forced splits
void oracle_get_diagnostics(void* h, int u, double* margins, int64_t* ties, int64_t* events) {
  const Unit& un = ((Oracle*)h)->units[u];
  if (margins) { margins[0] = un.mg.assign; margins[1] = un.mg.trigger; margins[2] = un.mg.select; margins[3] = un.mg.split; }
  if (ties) std::copy(un.ties, un.ties + 5, ties);
  if (events) { events[0] = un.n_splits; events[1] = un.n_failed_splits; events[2] = un.n_forced; }
}

}  // extern "C"
