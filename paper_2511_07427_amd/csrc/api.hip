// Host side of the C ABI declared in include/dynakv.h: argument checks, the carving of the caller's
// workspace into the arrays of `View`, and the kernel launches of every call.
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "common.hpp"

using namespace dynakv;

struct dynakv_index {
  dynakv_config_t cfg;
  View view;
  void* workspace;
  size_t bytes;
  bool built;
  int local_count;   // local update: appends enqueued since the last local clustering
  // optional timing of the gather + attention kernel
  bool profiling;
  std::vector<hipEvent_t> ev;   // start/stop pairs
  int n_prof;
  int prof_every = 1, prof_run = 1;   // of every prof_every launches the first prof_run are timed, as one bracket
  long long prof_seen = 0;            // launches since the last enable
};

namespace {

bool config_ok(const dynakv_config_t* c) {
  if (!c) return false;
  if (c->n_units < 1 || c->group_size < 1 || c->group_size > 16 || c->head_dim != kHeadDim) return false;
  if (c->dtype != DYNAKV_F32 && c->dtype != DYNAKV_F16 && c->dtype != DYNAKV_BF16) return false;
  if (c->n_clusters_init < 1 || c->n_clusters_init > kMaxInitClusters) return false;
  if (c->max_clusters < c->n_clusters_init || c->max_clusters > kMaxClusters) return false;
  if (c->max_tokens < c->n_clusters_init || c->max_tokens >= (1 << 22)) return false;
  if (c->kmeans_iters < 1 || c->buffer_max < 0) return false;
  if (c->group_reduce != DYNAKV_GROUP_MAX && c->group_reduce != DYNAKV_GROUP_SUM) return false;
  if (c->softmax_scale < 0.f) return false;
  if (c->search_copy != DYNAKV_SEARCH_STORAGE && c->search_copy != DYNAKV_SEARCH_MEAN) return false;
  if (c->score_round != 0 && c->score_round != 1) return false;
  if (c->update_mode < DYNAKV_UPDATE_ADAPTIVE || c->update_mode > DYNAKV_UPDATE_LOCAL) return false;
  if (c->update_mode == DYNAKV_UPDATE_LOCAL) {
    if (c->local_window < 2 || c->local_window > kLocalWindowMax) return false;
    if (c->local_clusters < 1 || c->local_clusters > kLocalClustersMax || c->local_clusters > c->local_window) return false;
  } else if (c->local_window != 0 || c->local_clusters != 0) {
    return false;
  }
  if (c->launch & ~(0xFFFF | DYNAKV_LAUNCH_SEPARATE | DYNAKV_LAUNCH_SPLIT_KERNEL)) return false;
  const int s = c->launch & 255, nw = (c->launch >> 8) & 255;
  if (s > kMaxKvSplits || (nw != 0 && nw != 4 && nw != 8 && nw != 16)) return false;
  return true;
}

int pow2_floor(int x) {
  int p = 1;
  while (2 * p <= x) p *= 2;
  return p;
}

// Shape of the gather + attention launch: S workgroups per unit of NW wavefronts each (the workgroup merge
// needs NW * G * 130 floats of LDS).  With S = 1 the single-kernel retrieval runs where it can.  Where it cannot
// (float32, more than kFusedClusters clusters or more than 8 query heads per unit) the separate kernels use one
// workgroup per unit from 32 units on: the step is bound by dependent round trips to memory rather than by the
// number of busy compute units, and every further workgroup per unit adds partial results, a ticket and a merge
// (measured on the 8-unit configuration: 4 workgroups per unit beat 1, 2, 8, 16 and 32; with 112 and 128 units
// 1 beats 2 and 3).  The configuration's `launch` field overrides both numbers.
void plan_attention(const dynakv_config_t& c, int* S, int* NW) {
  // split-KV (separate kernels): measured at 16384 + tokens per unit, budget 4096, with 1..128 units: 8 workgroups
  // per unit up to 32 units, then 256 / units (e.g. 16 units: 10.8k steps/s with 8, 9.5k with 2; 64 units: 7.6k with 4,
  // 6.1k with 1; more than 8 lose to the merge of the partial results)
  int s = (256 + c.n_units - 1) / c.n_units;
  if (s > 8) s = 8;
  // where the single-kernel retrieval can run (see retrieve_is_fused) it beats split-KV at every unit count:
  // measured 16.5k against 15.5k steps/s with 8 units, 15.1k against 13.1k with 24 (configuration 2's shape)
  if (c.dtype != DYNAKV_F32 && c.search_copy == DYNAKV_SEARCH_STORAGE && c.max_clusters <= kFusedClusters && c.group_size <= 8 &&
      c.update_mode != DYNAKV_UPDATE_TOKENS && c.update_mode != DYNAKV_UPDATE_LOCAL)
    s = 1;
  int nw = pow2_floor(4096 / (c.n_units * s) > 0 ? 4096 / (c.n_units * s) : 1);
  if (c.launch & 255) s = c.launch & 255;
  if ((c.launch >> 8) & 255) nw = (c.launch >> 8) & 255;
  const int lds_max = pow2_floor(65536 / (c.group_size * (kHeadDim + 2) * 4));
  nw = nw < 4 ? 4 : (nw > 16 ? 16 : pow2_floor(nw));
  if (nw > lds_max) nw = lds_max < 4 ? 4 : lds_max;
  if (c.group_size > 4 && nw > 8) nw = 8;    // 64 head rows fit the merge buffer of the single-kernel retrieval
  if (c.dtype == DYNAKV_F32) nw = 4;
  *S = s < 1 ? 1 : (s > kMaxKvSplits ? kMaxKvSplits : s);
  *NW = nw;
}

// Pages per unit: every token, one partly filled page per cluster, and room for a split to write both
// children before the parent's pages are recycled.
int pages_per_unit(const dynakv_config_t& c) {
  return (c.max_tokens + kPageTokens - 1) / kPageTokens + c.max_clusters + kMaxSplitMembers / kPageTokens + 2;
}

// Lays the arrays of `View` out in a workspace starting at `base` (may be null: size only).
size_t carve(const dynakv_config_t& c, char* base, View* out) {
  View v;
  std::memset(&v, 0, sizeof(v));
  v.U = c.n_units; v.G = c.group_size; v.dtype = c.dtype; v.M0 = c.n_clusters_init; v.Mcap = c.max_clusters;
  v.Ncap = c.max_tokens; v.Pcap = pages_per_unit(c); v.Lcap = (c.max_tokens + 3) & ~3; v.Bmax = c.buffer_max; v.group_reduce = c.group_reduce;
  plan_attention(c, &v.S, &v.NW);
  v.fuse = (c.launch & DYNAKV_LAUNCH_SEPARATE) ? 0 : (c.launch & DYNAKV_LAUNCH_SPLIT_KERNEL) ? 1 : 2;
  v.search_mean = c.dtype == DYNAKV_F32 || c.search_copy == DYNAKV_SEARCH_MEAN;
  v.score_round = c.score_round;
  v.static_update = c.update_mode == DYNAKV_UPDATE_STATIC;
  v.token_level = c.update_mode == DYNAKV_UPDATE_TOKENS || c.update_mode == DYNAKV_UPDATE_LOCAL;
  v.local_W = c.local_window; v.local_k = c.local_clusters;
  v.var_alpha = c.var_alpha; v.size_factor = c.size_factor;
  v.scale_d = c.softmax_scale > 0.f ? (double)c.softmax_scale : 1.0 / std::sqrt((double)c.head_dim);
  v.scale_f = (float)v.scale_d;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += (bytes + 255) & ~(size_t)255;
    return p;
  };
  const size_t U = v.U, UM = U * v.Mcap, UP = U * v.Pcap, UN = U * v.Ncap;
  v.search_mean = c.dtype == DYNAKV_F32 || c.search_copy == DYNAKV_SEARCH_MEAN;
  v.M = (int*)take(U * 4); v.N = (int*)take(U * 4); v.err = (int*)take(U * 4); v.tau = (double*)take(U * 8);
  v.nflag = (int*)take(U * 4); v.n_sel = (int*)take(U * 4); v.t_sel = (int*)take(U * 4); v.n_list = (int*)take(U * 4);
  v.ticket = (int*)take(U * 4); v.bump = (int*)take(U * 4); v.free_top = (int*)take(U * 4);
  v.NB = (v.Mcap + 255) / 256;
  v.near_d = (double*)take(U * v.NB * 8); v.near_j = (int*)take(U * v.NB * 4);
  v.zdist = (float*)take(v.search_mean ? 0 : UM * 4); v.rmax2 = (int*)take(U * 4); v.lcount = (int*)take(U * 4);
  const size_t nw = v.search_mean ? 0 : U * v.NB * 4;
  v.near_zb = (float*)take(nw * 4); v.near_z2 = (float*)take(nw * 4); v.near_zj = (int*)take(nw * 4);
  v.last_assign = (int*)take(U * 4); v.counters = (long long*)take(U * kCounters * 8);
  v.Rstride = r_stride(v.Mcap);
  v.R = (float*)take(U * v.Rstride * 4);
  v.Rq = (uint16_t*)take(c.dtype == DYNAKV_F32 ? 0 : U * v.Rstride * 2);
  v.cn = (int*)take(UM * 4); v.cb = (int*)take(UM * 4); v.csz = (int*)take(UM * 4); v.cflag = (int*)take(UM * 4); v.flist = (int*)take(UM * 4); v.cM2 = (double*)take(UM * 8);
  v.cpg = (int*)take(UM * kInlinePages * 4); v.ctail = (int*)take(UM * 4); v.score = (float*)take(UM * 4);
  v.sel_ids = (int*)take(UM * 4); v.in_req = (unsigned char*)take(UM); v.tok_off = (int*)take(UM * 4);
  v.pg_off = (int*)take(UM * 4);
  v.pages = take(UP * (size_t)kPageElems * elem_size(c.dtype));
  v.ppos = (int*)take(UP * kPageTokens * 4); v.pnext = (int*)take(UP * 4); v.freelist = (int*)take(UP * 4);
  v.plist = (int*)take(U * v.Lcap * 4); v.plist_off = (int*)take(U * v.Lcap * 4);
  v.part = (float*)take(U * v.S * v.G * (kHeadDim + 2) * 4);
  v.labels = (int*)take(UN * 4); v.order = (int*)take(UN * 4); v.dist = (double*)take(UN * 8);
  v.koff = (int*)take(U * (v.Mcap + 1) * 4);
  const size_t mpad = (size_t)((v.M0 + 31) / 32) * 32;
  v.kmA_stride = mpad * kHeadDim * 3;                    // up to three 16-bit terms per coordinate
  v.kmA = (uint16_t*)take(U * v.kmA_stride * 2);
  v.hn = (float*)take(U * mpad * 4); v.rmax = (float*)take(U * 4);
  v.nflagged = (int*)take(U * 4); v.has_empty = (int*)take(U * 4); v.xrange = (int*)take(U * 8);
  if (out) *out = v;
  return off;
}

}  // namespace

// An append where every entry becomes a cluster of its own; in local-update mode the window's clustering follows
// the append that fills it (the device keeps its own count and skips the clustering if an append was refused).
static dynakv_status_t append_own_cluster(dynakv_index* ix, const void* k, const void* val, hipStream_t st) {
  if (launch_append(ix->view, k, val, false, false, st) != hipSuccess) return DYNAKV_EHIP;
  if (ix->view.local_W > 0 && ++ix->local_count >= ix->view.local_W) {
    ix->local_count = 0;
    if (launch_local_recluster(ix->view, ix->cfg.kmeans_iters, st) != hipSuccess) return DYNAKV_EHIP;
  }
  return DYNAKV_OK;
}

extern "C" {

size_t dynakv_workspace_bytes(const dynakv_config_t* cfg) {
  if (!config_ok(cfg)) return 0;
  return carve(*cfg, nullptr, nullptr);
}

dynakv_status_t dynakv_create(const dynakv_config_t* cfg, void* workspace, size_t bytes, dynakv_index_t** out) {
  if (!out) return DYNAKV_EINVAL;
  *out = nullptr;
  if (!config_ok(cfg) || !workspace || ((uintptr_t)workspace & 255)) return DYNAKV_EINVAL;
  if (bytes < carve(*cfg, nullptr, nullptr)) return DYNAKV_ECAPACITY;
  dynakv_index* ix = new (std::nothrow) dynakv_index();
  if (!ix) return DYNAKV_ENOMEM;
  ix->cfg = *cfg;
  ix->workspace = workspace;
  ix->bytes = carve(*cfg, (char*)workspace, &ix->view);
  ix->built = false;
  ix->local_count = 0;
  ix->profiling = false;
  ix->n_prof = 0;
  *out = ix;
  return DYNAKV_OK;
}

dynakv_status_t dynakv_destroy(dynakv_index_t* ix) {
  if (!ix) return DYNAKV_EINVAL;
  for (hipEvent_t e : ix->ev) (void)hipEventDestroy(e);
  delete ix;
  return DYNAKV_OK;
}

dynakv_status_t dynakv_build_index(dynakv_index_t* ix, const void* K, const void* V, int32_t n_tokens,
                                   const int32_t* init_idx, void* stream) {
  if (!ix || !K || !V || !init_idx) return DYNAKV_EINVAL;
  if (n_tokens < ix->cfg.n_clusters_init || n_tokens > ix->cfg.max_tokens || n_tokens > kMaxPrefill) return DYNAKV_EINVAL;
  const hipError_t e = launch_build_index(ix->view, K, V, n_tokens, init_idx, ix->cfg.kmeans_iters, ix->workspace,
                                          ix->bytes, (hipStream_t)stream);
  if (e != hipSuccess) return DYNAKV_EHIP;
  ix->built = true;
  ix->local_count = 0;
  return DYNAKV_OK;
}

// Retrieval on the index as `view` shows it (the index's own view, or one whose scratch arrays point elsewhere),
// and with kin != null the append as well if one kernel can do both (*appended says whether it did), and with
// `split` the due splits too (*appended then covers them).
static dynakv_status_t retrieve_impl(dynakv_index_t* ix, const View& view, const void* Q, int32_t token_budget, float* out,
                                     float* lse, const void* kin, const void* vin, bool split, hipStream_t st,
                                     bool* appended) {
  const bool fused = retrieve_is_fused(view);
  *appended = fused && kin;
  if (!fused && launch_score_select(view, Q, token_budget, kin, st) != hipSuccess) return DYNAKV_EHIP;
  const int phase = ix->profiling ? (int)(ix->prof_seen++ % ix->prof_every) : -1;
  const bool prof = phase >= 0 && phase < ix->prof_run && 2 * (ix->n_prof + 1) <= (int)ix->ev.size();
  if (prof && phase == 0 && hipEventRecord(ix->ev[2 * ix->n_prof], st) != hipSuccess) return DYNAKV_EHIP;
  if (fused) {
    if (launch_retrieve_fused(view, Q, token_budget, out, lse, kin, vin, split, st) != hipSuccess) return DYNAKV_EHIP;
  } else if (launch_gather_attend(view, Q, out, lse, st) != hipSuccess) {
    return DYNAKV_EHIP;
  }
  if (prof) {
    if (phase == ix->prof_run - 1) {
      if (hipEventRecord(ix->ev[2 * ix->n_prof + 1], st) != hipSuccess) return DYNAKV_EHIP;
      ++ix->n_prof;
    }
  }
  return DYNAKV_OK;
}

dynakv_status_t dynakv_retrieve_attend(dynakv_index_t* ix, const void* Q, int32_t token_budget, float* out, float* lse,
                                       void* stream) {
  if (!ix || !Q || !out || token_budget < 0) return DYNAKV_EINVAL;
  if (!ix->built) return DYNAKV_ESTATE;
  bool appended;
  return retrieve_impl(ix, ix->view, Q, token_budget, out, lse, nullptr, nullptr, false, (hipStream_t)stream, &appended);
}

// ---- retrieval for callers that cannot allocate ---------------------------------------------------
// The scratch of the split-KV gather + attention (partial results of every workgroup and the arrival tickets)
// in a file-scope device array instead of the caller's workspace.  Each GPU holds its own copy of the array at
// its own address: the address is looked up once per device, with that device current, and kept.
constexpr size_t kStaticScratchBytes = DYNAKV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static hipError_t scratch_of_current_device(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = (unsigned char*)g_scratch_ptr[dev];
  return hipSuccess;
}

dynakv_status_t dynakv_retrieve_attend_static(dynakv_index_t* ix, const void* Q, int32_t token_budget, float* out,
                                              float* lse, void* stream) {
  if (!ix || !Q || !out || token_budget < 0) return DYNAKV_EINVAL;
  const View& v = ix->view;
  const size_t part_bytes = ((size_t)v.U * v.S * v.G * (kHeadDim + 2) * sizeof(float) + 255) & ~(size_t)255;
  const size_t ticket_bytes = (size_t)v.U * sizeof(int);
  if (part_bytes + ticket_bytes > kStaticScratchBytes) return DYNAKV_ECAPACITY;
  if (!ix->built) return DYNAKV_ESTATE;
  unsigned char* base = nullptr;
  if (scratch_of_current_device(&base) != hipSuccess) return DYNAKV_EHIP;
  View vs = v;                       // the kernels take the scratch as they take the workspace's: through the view
  vs.part = (float*)base;
  vs.ticket = (int*)(base + part_bytes);   // reset by the selection of this very call before any workgroup takes one
  bool appended;
  return retrieve_impl(ix, vs, Q, token_budget, out, lse, nullptr, nullptr, false, (hipStream_t)stream, &appended);
}

dynakv_status_t dynakv_decode_step(dynakv_index_t* ix, const void* Q, int32_t token_budget, float* out, float* lse,
                                   const void* k_new, const void* v_new, void* stream) {
  if (!ix || !Q || !out || token_budget < 0 || !k_new || !v_new) return DYNAKV_EINVAL;
  if (!ix->built) return DYNAKV_ESTATE;
  hipStream_t st = (hipStream_t)stream;
  bool appended;
  if (ix->view.token_level) {                        // no nearest-cluster search, no splits
    const dynakv_status_t rc = retrieve_impl(ix, ix->view, Q, token_budget, out, lse, nullptr, nullptr, false, st, &appended);
    if (rc != DYNAKV_OK) return rc;
    return append_own_cluster(ix, k_new, v_new, st);
  }
  const bool one_kernel = ix->view.fuse == 2;        // the splits too, where the retrieval kernel takes the append
  const dynakv_status_t rc = retrieve_impl(ix, ix->view, Q, token_budget, out, lse, k_new, v_new, one_kernel, st, &appended);
  if (rc != DYNAKV_OK) return rc;
  if (appended && one_kernel) return DYNAKV_OK;
  // separate kernels: the score kernel of this step has already looked for the new key's nearest cluster, and the
  // splits follow the append in its launch
  if (!appended) return launch_append(ix->view, k_new, v_new, true, true, st) == hipSuccess ? DYNAKV_OK : DYNAKV_EHIP;
  return launch_split(ix->view, st) == hipSuccess ? DYNAKV_OK : DYNAKV_EHIP;
}

dynakv_status_t dynakv_append(dynakv_index_t* ix, const void* k_new, const void* v_new, void* stream) {
  if (!ix || !k_new || !v_new) return DYNAKV_EINVAL;
  if (!ix->built) return DYNAKV_ESTATE;
  if (ix->view.token_level) return append_own_cluster(ix, k_new, v_new, (hipStream_t)stream);
  return launch_append(ix->view, k_new, v_new, false, false, (hipStream_t)stream) == hipSuccess ? DYNAKV_OK : DYNAKV_EHIP;
}

dynakv_status_t dynakv_extend_index(dynakv_index_t* ix, const void* K, const void* V, int32_t n_tokens, void* stream) {
  if (!ix || !K || !V || n_tokens < 1) return DYNAKV_EINVAL;
  if (!ix->built) return DYNAKV_ESTATE;
  if (ix->view.token_level) return DYNAKV_EINVAL;
  View v = ix->view;
  v.Bmax = 0;                                        // the chunk is resident: flagged clusters are split at once
  return launch_extend(v, K, V, n_tokens, (hipStream_t)stream) == hipSuccess ? DYNAKV_OK : DYNAKV_EHIP;
}

dynakv_status_t dynakv_place_by_coretrieval(dynakv_index_t* ix, const void* K, const void* V, int32_t n_tokens,
                                            const void* Qref, int32_t n_ref, int32_t token_budget, float* P,
                                            int32_t* order, void* stream) {
  if (!ix || !K || !V || !Qref || !P || n_ref < 1 || token_budget < 0) return DYNAKV_EINVAL;
  if (n_tokens < ix->cfg.n_clusters_init || n_tokens > ix->cfg.max_tokens) return DYNAKV_EINVAL;
  if (!ix->built) return DYNAKV_ESTATE;
  return launch_place(ix->view, K, V, n_tokens, Qref, n_ref, token_budget, P, order, (hipStream_t)stream) == hipSuccess
             ? DYNAKV_OK : DYNAKV_EHIP;
}

dynakv_status_t dynakv_split(dynakv_index_t* ix, void* stream) {
  if (!ix) return DYNAKV_EINVAL;
  if (!ix->built) return DYNAKV_ESTATE;
  if (ix->view.token_level || ix->view.static_update) return DYNAKV_OK;       // nothing is ever flagged
  return launch_split(ix->view, (hipStream_t)stream) == hipSuccess ? DYNAKV_OK : DYNAKV_EHIP;
}

dynakv_status_t dynakv_export_state(dynakv_index_t* ix, const dynakv_state_t* dst, void* stream) {
  if (!ix || !dst) return DYNAKV_EINVAL;
  if (!ix->built) return DYNAKV_ESTATE;
  hipStream_t st = (hipStream_t)stream;
  if (launch_export(ix->view, *dst, st) != hipSuccess) return DYNAKV_EHIP;
  // the sticky error words leave the device as a status here: this call waits for the stream
  std::vector<int> err((size_t)ix->view.U, 0);
  if (hipMemcpyAsync(err.data(), ix->view.err, err.size() * sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess) return DYNAKV_EHIP;
  if (hipStreamSynchronize(st) != hipSuccess) return DYNAKV_EHIP;
  for (int e : err)
    if (e) return DYNAKV_ECAPACITY;
  return DYNAKV_OK;
}

dynakv_status_t dynakv_import_state(dynakv_index_t* ix, const dynakv_state_t* src, void* stream) {
  if (!ix || !src) return DYNAKV_EINVAL;
  if (!src->n_clusters || !src->n_tokens || !src->tau || !src->centroids || !src->size || !src->buffered || !src->flag ||
      !src->m2 || !src->offsets || !src->members || !src->keys || !src->values)
    return DYNAKV_EINVAL;
  if ((src->n_selected == nullptr) != (src->selected == nullptr)) return DYNAKV_EINVAL;
  if (launch_import(ix->view, *src, (hipStream_t)stream) != hipSuccess) return DYNAKV_EHIP;
  ix->built = true;
  ix->local_count = 0;
  return DYNAKV_OK;
}

dynakv_status_t dynakv_profile_enable(dynakv_index_t* ix, int32_t max_launches) {
  if (!ix || max_launches < 0 || max_launches > (1 << 20)) return DYNAKV_EINVAL;
  while ((int)ix->ev.size() < 2 * max_launches) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return DYNAKV_EHIP;
    ix->ev.push_back(e);
  }
  ix->profiling = max_launches > 0;
  ix->n_prof = 0;
  ix->prof_seen = 0;
  return DYNAKV_OK;
}

dynakv_status_t dynakv_profile_sample(dynakv_index_t* ix, int32_t every, int32_t run) {
  if (!ix || every < 1 || run < 1 || run > every) return DYNAKV_EINVAL;
  ix->prof_every = every;
  ix->prof_run = run;
  return DYNAKV_OK;
}

dynakv_status_t dynakv_profile_read(dynakv_index_t* ix, int32_t* n_launches, double* total_ms) {
  if (!ix || !n_launches || !total_ms) return DYNAKV_EINVAL;
  double tot = 0.0;
  for (int i = 0; i < ix->n_prof; ++i) {
    if (hipEventSynchronize(ix->ev[2 * i + 1]) != hipSuccess) return DYNAKV_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ix->ev[2 * i], ix->ev[2 * i + 1]) != hipSuccess) return DYNAKV_EHIP;
    tot += ms;
  }
  *n_launches = ix->n_prof * ix->prof_run;       // launches inside completed brackets
  *total_ms = tot;
  return DYNAKV_OK;
}

const char* dynakv_profiled_kernel(dynakv_index_t* ix) {
  return ix && retrieve_is_fused(ix->view) ? "retrieve_fused_kernel" : "gather_attend_kernel";
}

const char* dynakv_strerror(dynakv_status_t s) {
  switch (s) {
    case DYNAKV_OK: return "ok";
    case DYNAKV_EINVAL: return "invalid argument or unsupported size";
    case DYNAKV_ECAPACITY: return "capacity exhausted: workspace or static scratch too small, or a unit's error word is set (tokens, clusters, pages)";
    case DYNAKV_ESTATE: return "call out of order: build the index first";
    case DYNAKV_EHIP: return "HIP runtime error";
    case DYNAKV_ENOMEM: return "out of host memory";
  }
  return "unknown status";
}

}  // extern "C"
