/* dynakv.h - C ABI of the MI355X (gfx950) library for cluster-indexed sparse attention over an
 * HBM-resident KVCache, following the adaptive KVCache management of the DynaKV paper
 * (Section 4: problem formulation Eq. 1-5, Algorithm 1, Section 4.2; k-means and the
 * overflow-safe attention over reordered KV of Section 7).
 *
 * One index holds U independent units (one per layer x sequence x KV head).  Per unit it keeps the
 * partition of the KVCache into clusters (Eq. 3), one float32 centroid per cluster (Eq. 4), the
 * per-cluster state of Algorithm 1 (size n_j, M2_j = n_j * variance, buffer count |Buf_j|, split
 * flag f_j), the head-specific threshold tau, and the keys/values themselves in cluster-contiguous
 * pages of 16 tokens.
 *
 * Conventions for every call
 *   memory    - every pointer marked "device" is device memory owned by the caller (in practice a
 *               torch tensor).  The library allocates no device memory and frees none; all of its
 *               state lives in the caller's workspace, which must outlive the handle.  Pointers
 *               marked "host" are ordinary host memory.
 *   streams   - `stream` is a hipStream_t (null = default stream).  Work is enqueued there and the
 *               call returns without waiting; inputs and outputs must stay valid until the stream
 *               has passed the call.  One handle is driven from one stream at a time.
 *   errors    - host-detectable misuse returns a status and enqueues nothing.  Conditions only
 *               the device can see (token, cluster or page capacity exhausted, invalid initial
 *               positions or imported state) set a sticky per-unit error word; the offending
 *               operation leaves the unit's state unchanged (a split that has no room leaves its
 *               cluster flagged); dynakv_export_state, which waits for the stream, reports the
 *               words and returns DYNAKV_ECAPACITY if any is set.
 *   numerics  - the statistics (mean, M2, threshold test) and the 2-means of a split are float64
 *               computations on the stored values.  With 16-bit storage, cluster scores and the
 *               distances of a new entry are first computed on the matrix cores (products of two
 *               16-bit values are exact, the 128 of them are accumulated in float32); every
 *               decision that the float32 rounding could change is then retaken on float64 values:
 *               the nearest cluster among all candidates within the error bound of the best, and
 *               the budget cut among all clusters whose score lies within the bound of the cut.
 *               The selected set therefore is the one of exact arithmetic; the order in which the
 *               selected clusters are attended is the library's own (ascending id; descending
 *               float32 score where max_clusters > 16384).  Ties go to the lowest index.
 *               Attention uses matrix cores with float32 accumulation.
 */
#ifndef DYNAKV_H
#define DYNAKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dynakv_index dynakv_index_t; /* opaque host-side handle */

typedef enum {
  DYNAKV_OK = 0,
  DYNAKV_EINVAL = 1,    /* bad argument or unsupported size */
  DYNAKV_ECAPACITY = 2, /* workspace or static scratch too small; from dynakv_export_state: a unit's error word is set */
  DYNAKV_ESTATE = 3,    /* call out of order (decode call before dynakv_build_index) */
  DYNAKV_EHIP = 4,      /* a HIP runtime call failed */
  DYNAKV_ENOMEM = 5     /* host memory for the handle could not be allocated */
} dynakv_status_t;

typedef enum { DYNAKV_F32 = 0, DYNAKV_F16 = 1, DYNAKV_BF16 = 2 } dynakv_dtype_t;
typedef enum { DYNAKV_GROUP_MAX = 0, DYNAKV_GROUP_SUM = 1 } dynakv_group_reduce_t;
/* Which copy of a centroid the two searches of a step read (query similarity, nearest cluster of the new entry;
 * Section 4.1, Algorithm 1: the paper fixes no precision).  STORAGE: the mean rounded to the type of the keys, like
 * the entries it stands for (half the bytes to scan; the float32 mean stays the master copy for the statistics).
 * MEAN: the float32 mean itself, scored in float64 on the vector units.  float32 storage always reads the mean. */
typedef enum { DYNAKV_SEARCH_STORAGE = 0, DYNAKV_SEARCH_MEAN = 1 } dynakv_search_copy_t;
/* ADAPTIVE: Algorithm 1.  STATIC: the static-update baseline of Section 2.3: entries join their nearest cluster
 * and update its statistics, no cluster is ever flagged or split.  TOKENS: the baseline without clustering of
 * Section 8.1: every appended entry becomes a cluster of its own (build the index with n_clusters_init = n_tokens
 * and init_idx = 0..n_tokens-1), so that the retrieval is an exact top-B over tokens; needs max_clusters >=
 * max_tokens (an append beyond it is refused with DYNAKV_ERR_CLUSTERS).  LOCAL: the local-update baseline of
 * Section 2.3: new entries are clustered among themselves, apart from the existing clusters: each is a cluster of
 * its own until local_window of them have come in; Lloyd's k-means over those (initial centres: every
 * (local_window / local_clusters)-th of them, kmeans_iters iterations, a centre without members stays where it is)
 * then replaces them by local_clusters clusters, which take the ids of the first of them.  The prefill's clusters
 * never change.  Needs max_clusters >= n_clusters_init + local_window + local_clusters * (appends / local_window). */
typedef enum {
  DYNAKV_UPDATE_ADAPTIVE = 0, DYNAKV_UPDATE_STATIC = 1, DYNAKV_UPDATE_TOKENS = 2, DYNAKV_UPDATE_LOCAL = 3
} dynakv_update_mode_t;

/* bits of the per-unit device error word */
#define DYNAKV_ERR_TOKENS 1   /* append refused: max_tokens or page pool exhausted            */
#define DYNAKV_ERR_CLUSTERS 2 /* split refused: max_clusters reached (cluster stays flagged)   */
#define DYNAKV_ERR_SPLIT_SIZE 4 /* split refused: cluster larger than the split kernel handles */
#define DYNAKV_ERR_SELECT 8   /* retrieval cut short: max_clusters > 16384 and more than 4096 clusters selected */
#define DYNAKV_ERR_INIT 16    /* dynakv_build_index: an initial position out of range or given twice */
#define DYNAKV_ERR_IMPORT 32  /* dynakv_import_state: inconsistent sizes; the unit keeps its previous state */
#define DYNAKV_ERR_PLACE 64   /* dynakv_place_by_coretrieval: the unit is not as dynakv_build_index left it; not re-placed */

/* Launch shape (dynakv_config_t.launch).  0 lets the library choose.  Otherwise the low byte is the number of
 * workgroups that share one unit's gather + attention (split-KV), the next byte their wavefronts (4, 8 or 16),
 * either 0 = chosen by the library, plus the flags below.  Results do not depend on the shape beyond float32
 * rounding of the attention output. */
#define DYNAKV_LAUNCH(kv_splits, att_waves) (((kv_splits) & 255) | (((att_waves) & 255) << 8))
#define DYNAKV_LAUNCH_SEPARATE (1 << 16)     /* scores, selection, gather + attention, append, split as separate kernels */
#define DYNAKV_LAUNCH_SPLIT_KERNEL (1 << 17) /* a whole-step call runs its splits in a kernel of their own */

typedef struct {
  int32_t n_units;         /* U >= 1                                                            */
  int32_t group_size;      /* G, query heads per KV head, 1..16                                 */
  int32_t head_dim;        /* d; must be 128                                                    */
  int32_t dtype;           /* dynakv_dtype_t of K, V and Q                                      */
  int32_t n_clusters_init; /* M0, clusters built at prefill                                     */
  int32_t max_clusters;    /* capacity per unit, splits included; M0..131072                     */
  int32_t max_tokens;      /* capacity per unit                                                 */
  int32_t kmeans_iters;    /* Lloyd iterations at prefill, >= 1, no early exit                  */
  int32_t buffer_max;      /* B_max of Algorithm 1; 0 = every cluster counts as resident        */
  int32_t group_reduce;    /* dynakv_group_reduce_t: how G head scores become one cluster score */
  float var_alpha;         /* tau = var_alpha * (k-means objective / N0) per unit; <= 0: off    */
  float size_factor;       /* also flag when n' > size_factor * (N+1)/M; <= 0: off              */
  float softmax_scale;     /* 0 = 1/sqrt(head_dim)                                              */
  int32_t search_copy;     /* dynakv_search_copy_t                                              */
  int32_t score_round;     /* 1: where the budget cut is retaken on float64 scores, they are rounded to
                              float32 first (equal float32 scores then go by id); 0: compared as float64 */
  int32_t update_mode;     /* dynakv_update_mode_t                                              */
  int32_t launch;          /* 0, or DYNAKV_LAUNCH(..) | DYNAKV_LAUNCH_* flags                    */
  int32_t local_window;    /* DYNAKV_UPDATE_LOCAL: entries per local clustering, 2..128; else 0  */
  int32_t local_clusters;  /* DYNAKV_UPDATE_LOCAL: clusters it forms, 1..min(32, local_window); else 0 */
} dynakv_config_t;

/* Bytes of device workspace an index of this configuration needs (0 if the configuration is invalid). */
size_t dynakv_workspace_bytes(const dynakv_config_t* cfg);

/* Creates the host-side handle over `workspace` (device, `bytes` long, 256-byte aligned).  Nothing is
 * enqueued; the workspace is initialised by dynakv_build_index.  EINVAL / ECAPACITY on bad input. */
dynakv_status_t dynakv_create(const dynakv_config_t* cfg, void* workspace, size_t bytes, dynakv_index_t** out);

/* Frees the host-side handle only. */
dynakv_status_t dynakv_destroy(dynakv_index_t* index);

/* Prefill (Algorithm 1, prefill block; Section 4.1 Eq. 3-4): Lloyd's k-means of each unit's keys into M0
 * clusters, then n_j, r_j, M2_j, tau, empty buffers and flags, and the cluster-contiguous page layout.
 *   K, V      device, [U][n_tokens][head_dim] in cfg.dtype, contiguous; read only
 *   n_tokens  M0 <= n_tokens <= min(max_tokens, 16384)
 *   init_idx  device, int32 [U][M0]: positions of the M0 distinct keys used as initial centres (a position out of
 *             range or given twice sets DYNAKV_ERR_INIT; the build then runs with the position clamped)
 * Empty clusters are re-seeded with the points farthest from their centres in every iteration but the
 * last.  Resets any earlier state of the index, error words included. */
dynakv_status_t dynakv_build_index(dynakv_index_t* index, const void* K, const void* V, int32_t n_tokens,
                                   const int32_t* init_idx, void* stream);

/* Adaptive clustering applied continuously through a long prefill (Section 7, Discussion 1): instead of one k-means
 * over the whole prompt (whose keys must all be resident at once), the index is built from the first chunk and
 * every further chunk is added with this call: its entries go through Algorithm 1's decode block one after the
 * other (nearest cluster, UpdateVar, threshold test), and because the chunk is resident a flagged cluster is
 * split at once (as with buffer_max = 0), whatever the configured buffer.  The active set is not consulted.
 *   K, V      device, [U][n_tokens][head_dim] in cfg.dtype, contiguous; read only
 *   n_tokens  >= 1; tokens beyond max_tokens are refused with DYNAKV_ERR_TOKENS
 * One kernel: each unit's workgroup walks its chunk in order. */
dynakv_status_t dynakv_extend_index(dynakv_index_t* index, const void* K, const void* V, int32_t n_tokens, void* stream);

/* Correlation-aware placement (Section 5.1, inter-cluster correlation, Eq. 8), kept here as a page-placement hint:
 * once, right after dynakv_build_index, n_ref reference retrievals (scores and budget cut only) count how often
 * two clusters are selected together, f(C_i, C_j) for i != j; P(ij) = f(C_i, C_j) / sum over all ordered pairs;
 * the clusters are then chained greedily (start: largest total count; next: the cluster co-selected most often
 * with the last one; lowest id among equals) and their pages are laid out afresh in that order, so that clusters
 * which tend to be retrieved together sit next to each other in the page pool.  Nothing else changes: partition,
 * statistics and retrieval results are the same as before (the active set is left as the last reference query
 * selected it).
 *   K, V        device, the arrays that were given to dynakv_build_index, [U][n_tokens][head_dim]
 *   Qref        device, [n_ref][U][G][head_dim] in cfg.dtype: the reference queries (the initial input)
 *   P           device, float32 [U][M0][M0]: receives Eq. 8's probabilities (used as the counting matrix meanwhile)
 *   order       device, int32 [U][M0] or null: receives the chain
 * A unit that has changed since it was built (appends, splits) is left alone and gets DYNAKV_ERR_PLACE. */
dynakv_status_t dynakv_place_by_coretrieval(dynakv_index_t* index, const void* K, const void* V, int32_t n_tokens,
                                            const void* Qref, int32_t n_ref, int32_t token_budget, float* P,
                                            int32_t* order, void* stream);

/* One retrieval (Algorithm 1, decode block: the top clusters by query-centroid similarity are loaded;
 * Section 4.1) followed by softmax attention over the retrieved entries (Section 7, attention over reordered KV):
 * score_j = scale * reduce_g <q_g, r~_j>, r~_j = the copy of the centroid selected by cfg.search_copy;
 * clusters are taken in (score desc, id asc) order while
 * their stored sizes n_j + |Buf_j| fit in `token_budget`, stopping at the first that does not fit; if
 * even the best cluster does not fit, its first `token_budget` entries are taken.  The selected set
 * becomes the active set P_req that dynakv_split consults.
 *   Q     device, [U][G][head_dim] in cfg.dtype
 *   out   device, float32 [U][G][head_dim]: softmax(scale * q K_sel^T) V_sel; zeros if nothing is selected
 *   lse   device, float32 [U][G] or null: log-sum-exp of the scaled logits (-inf if nothing is selected)
 * The new token of the step is not part of the index yet; merge it through `lse` if needed. */
dynakv_status_t dynakv_retrieve_attend(dynakv_index_t* index, const void* Q, int32_t token_budget, float* out,
                                       float* lse, void* stream);

/* dynakv_retrieve_attend for callers that cannot allocate device memory or hand over a workspace region for
 * scratch (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and results, but the scratch of the split-KV gather + attention (every workgroup's partial sums,
 * maxima and accumulators, and the arrival tickets of each unit) lives in a device array inside the library
 * of DYNAKV_STATIC_SCRATCH_BYTES, which every GPU the library runs on holds until the process ends.  The call
 * allocates nothing.  It needs n_units * kv_splits * group_size * 130 * 4 + n_units * 4 bytes; a configuration
 * that needs more returns DYNAKV_ECAPACITY and enqueues nothing.  All calls on one GPU share the array: calls
 * that overlap on one GPU (two streams, two indexes) race; what must start at zero is cleared by the call itself.
 * Arguments as dynakv_retrieve_attend. */
#define DYNAKV_STATIC_SCRATCH_BYTES (8u << 20)
dynakv_status_t dynakv_retrieve_attend_static(dynakv_index_t* index, const void* Q, int32_t token_budget, float* out,
                                              float* lse, void* stream);

/* Adds one entry per unit (Algorithm 1, decode block: assign to the nearest cluster (squared distance to r~_j, see
 * dynakv_retrieve_attend), UpdateVar on the float32 mean, threshold test, then
 * AddEntry + UpdateStats or buffer + flag; Section 4.2).  The entry is always stored at the tail of its
 * cluster's pages; a cluster whose tentative variance exceeds tau (or whose tentative size exceeds the
 * size trigger) is flagged and keeps its statistics frozen, later entries of a flagged cluster count as
 * buffered.
 *   k_new, v_new  device, [U][head_dim] in cfg.dtype */
dynakv_status_t dynakv_append(dynakv_index_t* index, const void* k_new, const void* v_new, void* stream);

/* Algorithm 1, delayed cluster splitting: splits every flagged cluster that the last retrieval selected
 * (all flagged clusters if buffer_max = 0), in ascending id; then, if the buffers together hold at least
 * buffer_max entries, also the flagged cluster with the most buffered entries.  A split is a 2-means of
 * the cluster's keys (seeds: the member farthest from the mean, then the member farthest from that one;
 * at most 16 Lloyd rounds); the child holding the earliest entry keeps the id, the other takes the next
 * free id; both get exact statistics.  A cluster that cannot be split (fewer than 2 entries, or all
 * equal) is unflagged with exact statistics. */
dynakv_status_t dynakv_split(dynakv_index_t* index, void* stream);

/* One whole decode step of Algorithm 1 (decode block): dynakv_retrieve_attend(Q), dynakv_append(k_new,
 * v_new) and dynakv_split(), in that order and with the same results bit for bit, so the three calls and
 * this one can be mixed freely.  It exists because the step's two passes over the centroid table (query
 * similarity, Section 4.1; nearest cluster of the new key, Section 4.2) read the same data, and because a
 * step is a chain of short dependent phases: with 16-bit storage read through its 16-bit search copy, at most
 * 4096 clusters and at most 8 query heads per unit the whole step is ONE kernel launch that reads the table
 * once, commits the append before it streams the selected pages, and prepares the due splits while it streams
 * them.  Otherwise (float32 storage or search copy, more clusters, more query heads) it is four launches
 * instead of the six of the three calls: the score kernel also evaluates the new key's distances, and the
 * splits run in the append's launch.  Arguments as in the three calls. */
dynakv_status_t dynakv_decode_step(dynakv_index_t* index, const void* Q, int32_t token_budget, float* out,
                                   float* lse, const void* k_new, const void* v_new, void* stream);

/* Snapshot of an index, written by dynakv_export_state and read by dynakv_import_state.  Every field is a device
 * pointer or null (null = skip). */
typedef struct {
  int32_t* n_clusters;   /* [U]                 M_t                                              */
  int32_t* n_tokens;     /* [U]                 N_t                                              */
  int32_t* error;        /* [U]                 DYNAKV_ERR_* bits                                */
  double* tau;           /* [U]                                                                  */
  float* centroids;      /* [U][max_clusters][head_dim]                                          */
  int32_t* size;         /* [U][max_clusters]   n_j                                              */
  int32_t* buffered;     /* [U][max_clusters]   |Buf_j|                                          */
  int32_t* flag;         /* [U][max_clusters]   f_j                                              */
  double* m2;            /* [U][max_clusters]   M2_j                                             */
  int32_t* offsets;      /* [U][max_clusters+1] members of cluster j: members[offsets[j]..offsets[j+1]) */
  int32_t* members;      /* [U][max_tokens]     token positions in storage order                 */
  float* scores;         /* [U][max_clusters]   scores of the last retrieval                     */
  int32_t* n_selected;   /* [U]                 clusters selected by the last retrieval          */
  int32_t* selected;     /* [U][max_clusters]   their ids in the order they are attended: ascending id
                                                (descending score where max_clusters > 16384)     */
  int32_t* n_gathered;   /* [U]                 entries attended by the last retrieval           */
  int32_t* gathered;     /* [U][max_tokens]     their token positions in gather order            */
  int32_t* last_assign;  /* [U]                 cluster chosen by the last append                */
  int64_t* counters;     /* [U][8]              splits, failed splits, forced splits, pages in use,
                                                entries gathered, retrievals, clusters scored,
                                                decisions retaken in float64 (all since build_index) */
  void* keys;            /* [U][max_tokens][head_dim] in cfg.dtype: key of every token, by position      */
  void* values;          /* [U][max_tokens][head_dim] in cfg.dtype: value of every token, by position    */
  int32_t* first_page;   /* [U][max_clusters]   first page of cluster j in the unit's page pool (-1: none);
                                                export only                                      */
} dynakv_state_t;

/* Copies the requested parts of the state, waits for `stream`, and returns DYNAKV_ECAPACITY if the error word of
 * any unit is set (the copy is complete in that case too), DYNAKV_OK otherwise. */
dynakv_status_t dynakv_export_state(dynakv_index_t* index, const dynakv_state_t* dst, void* stream);

/* Replaces the whole state of the index by a snapshot (Algorithm 1's state: the partition, n_j, r_j, M2_j, Buf_j,
 * f_j, tau, and the active set P_req of the last retrieval), e.g. one that dynakv_export_state wrote, so that a
 * run can be resumed or continued elsewhere.  Required fields: n_clusters, n_tokens, tau, centroids, size,
 * buffered, flag, m2, offsets, members, keys, values; optional: n_selected with selected (else the active set is
 * empty).  The other fields are ignored.  Pages are laid out afresh, cluster by cluster; error words and counters
 * start at zero.  A unit whose sizes are inconsistent (cluster or token count beyond capacity, offsets that do
 * not match size + buffered) keeps its previous state and gets DYNAKV_ERR_IMPORT.  Counts as building the index. */
dynakv_status_t dynakv_import_state(dynakv_index_t* index, const dynakv_state_t* src, void* stream);

/* Timing aid: when enabled, the dominant kernel of dynakv_retrieve_attend / dynakv_decode_step (gather +
 * attention; where it can run, the single kernel that also scores and selects and, in a decode step,
 * appends and splits) is bracketed by HIP events on its own stream.  dynakv_profile_read synchronises those events and
 * returns the number of launches and their summed duration in milliseconds since the last enable. */
dynakv_status_t dynakv_profile_enable(dynakv_index_t* index, int32_t max_launches);
/* Two events around a launch cost the stream several microseconds between kernels and are themselves inside
 * what they measure.  With every > 1 only the launches k (counted from the last enable) with k % every < run are
 * timed, each such run of consecutive launches inside ONE bracket: an even sample of the whole run of calls.
 * dynakv_profile_enable's max_launches then counts brackets, and dynakv_profile_read returns the launches inside
 * completed brackets with their summed duration.  run > 1 is meant for dynakv_decode_step where the step is one
 * kernel: whatever else the stream executes between the launches of a run lies inside the bracket.
 * every < 1, run < 1 or run > every: DYNAKV_EINVAL.  Stays in force until set again; (1, 1) at creation. */
dynakv_status_t dynakv_profile_sample(dynakv_index_t* index, int32_t every, int32_t run);
dynakv_status_t dynakv_profile_read(dynakv_index_t* index, int32_t* n_launches, double* total_ms);
/* Name of the kernel those events bracket: "retrieve_fused_kernel" (scores + selection + gather + attention in
 * one launch; in dynakv_decode_step the append and the splits as well) or "gather_attend_kernel". */
const char* dynakv_profiled_kernel(dynakv_index_t* index);

const char* dynakv_strerror(dynakv_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* DYNAKV_H */
