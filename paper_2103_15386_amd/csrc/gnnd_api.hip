// Host side of the C ABI declared in include/gnnd.h: argument validation,
// workspace layout, stage sequencing, statistics.  No device memory is
// allocated here; every array is carved out of the caller's workspace.
#include <hip/hip_runtime.h>

#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <atomic>
#include <cerrno>
#include <chrono>
#include <cstdio>
#include <deque>
#include <mutex>
#include <cstring>
#include <new>
#include <string>
#include <thread>
#include <utility>
#include <vector>

#include "../../include/gnnd.h"
#include "device_utils.hpp"
#include "kernels.hpp"

using namespace gnnd;

// Workspace of gnnd_build_static: one array per GPU, part of the loaded code
// object, so the entry point needs no allocation.  Host code never uses this
// name as an address; it asks the runtime for the array's device address once
// per device (static_scratch_of) and passes that pointer on.
constexpr size_t kStaticScratchBytes = GNND_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_last_error = "";

struct Layout {
  size_t off_G, off_kth, off_snew, off_sold, off_cnew, off_cold, off_ron,
      off_roo, off_csn, off_cso, off_capn, off_capo, off_pslot, off_poff, off_bins, off_scan,
      off_cnt, off_snap, off_aside, off_shadow, off_norms, off_flag, off_bkc, off_bko, off_stg_ent,
      off_stg_cur, off_cls_nodes, off_cls_count, total;
};

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

const char* check_params(const gnnd_params* q) {
  if (!q) return "params is NULL";
  if (q->metric < GNND_L2SQ_F32 || q->metric > GNND_COSINE_F32) return "unknown metric";
  if (q->k < 2 || q->k > 128) return "k must be in [2, 128]";
  if (q->p < 1 || q->p > 64 || q->p > q->k) return "p must be in [1, min(k, 64)]";
  if (q->d < 1) return "d must be >= 1";
  if (q->metric == GNND_L2SQ_U8 && q->d > 32768) return "d must be <= 32768 for uint8 vectors";
  if (q->n <= q->k) return "n must exceed k";
  if (q->n > ((int64_t)1 << 27)) return "n must be <= 2^27";
  if (q->n * (int64_t)q->p >= ((int64_t)1 << 32)) return "n * p must be below 2^32";
  if (q->join_path < GNND_JOIN_AUTO || q->join_path > GNND_JOIN_GRAM) return "unknown join_path";
  if (q->update_mode != GNND_UPDATE_SELECTIVE && q->update_mode != GNND_UPDATE_ALL_PAIRS)
    return "unknown update_mode";
  if (q->update_mode == GNND_UPDATE_ALL_PAIRS &&
      (q->join_path == GNND_JOIN_MFMA || q->join_path == GNND_JOIN_MFMA_DIRECT ||
       q->join_path == GNND_JOIN_GRAM))
    return "GNND_UPDATE_ALL_PAIRS runs with GNND_JOIN_VALU (or GNND_JOIN_AUTO) only";
  if (q->update_mode == GNND_UPDATE_ALL_PAIRS && q->p > 32)
    return "GNND_UPDATE_ALL_PAIRS needs p <= 32";
  if (q->join_path == GNND_JOIN_GRAM &&
      (q->p > 32 || (q->metric != GNND_L2SQ_F32 && q->metric != GNND_ANGULAR_F32 &&
                     q->metric != GNND_COSINE_F32)))
    return "GNND_JOIN_GRAM needs float32 vectors, p <= 32 and the squared-L2, angular or cosine "
           "metric";
  if (q->list_mode != GNND_LISTS_PLAIN && q->list_mode != GNND_LISTS_SEGMENTED)
    return "unknown list_mode";
  if (q->list_mode == GNND_LISTS_SEGMENTED) {
    if (q->k % 32 != 0) return "segmented lists need k = 32, 64, 96 or 128";
    if (q->n < (int64_t)34 * (q->k / 32))
      return "segmented lists need n >= 34 k / 32 (more than 32 other objects per residue class)";
    if (q->update_mode != GNND_UPDATE_SELECTIVE) return "segmented lists run the selective update";
  }
  return nullptr;
}

// The matrix-core join handles byte-valued data of up to 128 dimensions: uint8
// vectors, or float32 vectors that turn out to hold only integers 0..255.
bool mfma_possible(const gnnd_params* q) {
  return q->join_path != GNND_JOIN_VALU && q->join_path != GNND_JOIN_GRAM &&
         q->update_mode == GNND_UPDATE_SELECTIVE && q->d <= 128 && q->p <= 32 &&
         (q->metric == GNND_L2SQ_U8 || q->metric == GNND_L2SQ_F32);
}

// The float32 matrix-core join (inner products by matrix instructions, canonical distances
// for the results) takes any float32 data under the metrics that are functions of an inner
// product and the norms.  Left to itself the library takes it wherever it applies: measured
// against the general join it is 10 to 16 % ahead on 96-, 128- and 960-dimensional data.
bool gram_possible(const gnnd_params* q) {
  return (q->join_path == GNND_JOIN_GRAM || q->join_path == GNND_JOIN_AUTO) &&
         q->update_mode == GNND_UPDATE_SELECTIVE && q->p <= 32 &&
         (q->metric == GNND_L2SQ_F32 || q->metric == GNND_ANGULAR_F32 ||
          q->metric == GNND_COSINE_F32);
}
bool needs_norms(const gnnd_params* q) {
  return q->metric == GNND_COSINE_F32 || gram_possible(q);
}

// The matrix-core join stages its results per bucket of destinations (instead of handing
// them on one by one) for up to 2^20 nodes: a staged result then fits one 64-bit word, and
// the staging array is as large again as the proposal array.
bool stage_possible(const gnnd_params* q) {
  return mfma_possible(q) && q->join_path != GNND_JOIN_MFMA_DIRECT && q->n <= kStageMaxNodes;
}

Layout make_layout(const gnnd_params* q, bool with_aside) {
  Layout L;
  const size_t n = (size_t)q->n, k = (size_t)q->k, p = (size_t)q->p;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes);
    return at;
  };
  L.off_G = take(n * k * 8);
  L.off_kth = take(n * sizeof(NodeMeta));
  L.off_snew = take(n * 2 * p * 4);
  L.off_sold = take(n * 2 * p * 4);
  L.off_cnew = take(n * 4);
  L.off_cold = take(n * 4);
  L.off_ron = take((n + 1) * 8);
  L.off_roo = take((n + 1) * 8);
  L.off_csn = take(n * p * 4);
  L.off_cso = take(n * p * 4);
  L.off_capn = take(n * 4);
  L.off_capo = take(n * 4);
  L.off_pslot = take(n * 8);
  L.off_poff = take((n + 1) * 8);
  const size_t slots_per_node =
      q->update_mode == GNND_UPDATE_ALL_PAIRS ? 2 * p * (6 * p - 1) : 6 * p;
  L.off_bins = take(n * slots_per_node * 8);
  L.off_scan = take(scan_tmp_elems((int64_t)n) * 8);
  L.off_cnt = take((size_t)kStripes * C_SLOTS * 8);
  L.off_snap = take((size_t)kStripes * C_SLOTS * 8);
  L.off_aside = take(with_aside ? n * (k / 2) * 8 : 0);
  const bool shadow = mfma_possible(q);
  L.off_shadow = take(shadow ? n * (size_t)((q->d + 31) & ~31) : 0);
  L.off_norms = take(needs_norms(q) ? n * 4 : 0);  // squared norms
  L.off_flag = take(256);
  L.off_bkc = take(2 * 4096 * 4);
  L.off_bko = take(2 * 4097 * 8);
  const bool staged = stage_possible(q);
  L.off_stg_ent = take(staged ? n * slots_per_node * 8 : 0);
  L.off_stg_cur = take(staged ? (size_t)kStageBuckets * 8 : 0);
  const bool gram = gram_possible(q);
  // (the float join lists its nodes in kGramClasses classes, the staged int8 join in three)
  L.off_cls_nodes = take(gram ? (size_t)kGramClasses * n * 4 : staged ? (size_t)3 * n * 4 : 0);
  L.off_cls_count = take(gram || staged ? 256 : 0);
  L.total = o;
  return L;
}

}  // namespace

constexpr int kProfItersDefault = 64;    // window of gnnd_set_profiling(ctx, 1)
constexpr int kProfItersMax = 1 << 16;   // largest window a caller may ask for
constexpr int kProfEvents = 5;  // before sampling, join, hand-out pass, update; after the update

struct gnnd_ctx {
  gnnd_params prm;
  Shape sh;
  DevState ds;
  hipStream_t stream;
  int32_t iter;       // iterations completed
  int stage;          // 0 = ready for sample, 1 = sampled, 2 = joined
  bool has_graph;
  bool fresh_random;  // the graph is what gnnd_init_random left: no update has touched it yet
  bool merge_mode;
  bool use_mfma;
  bool use_gram;
  int* flag_dev;
  hipEvent_t ev[5];
  bool have_events;
  // profiling mode: four events per iteration, recorded without synchronising
  bool prof_on;
  int prof_count;   // iterations recorded in the current window
  int prof_missed;  // iterations that found the window full (not recorded)
  std::vector<hipEvent_t> prof;  // kProfEvents events per iteration of the window
  uint64_t* snap;  // device copy of the counters taken when the iteration began
  std::string err;
};

namespace {

int fail(gnnd_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  g_last_error = msg;
  return code;
}
int hip_fail(gnnd_ctx* c, hipError_t e, const char* what) {
  return fail(c, GNND_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

void bind(gnnd_ctx* c, const Layout& L) {
  char* w = (char*)c->prm.workspace_dev;
  DevState& d = c->ds;
  d.G = (uint64_t*)(w + L.off_G);
  d.meta = (NodeMeta*)(w + L.off_kth);
  d.snew = (int32_t*)(w + L.off_snew);
  d.sold = (int32_t*)(w + L.off_sold);
  d.cnew = (int32_t*)(w + L.off_cnew);
  d.cold = (int32_t*)(w + L.off_cold);
  d.roff_new = (uint64_t*)(w + L.off_ron);
  d.roff_old = (uint64_t*)(w + L.off_roo);
  d.csr_new = (int32_t*)(w + L.off_csn);
  d.csr_old = (int32_t*)(w + L.off_cso);
  d.pslot = (uint64_t*)(w + L.off_pslot);
  d.poff = (uint64_t*)(w + L.off_poff);
  d.capn = (uint32_t*)(w + L.off_capn);
  d.capo = (uint32_t*)(w + L.off_capo);
  d.bins = (uint64_t*)(w + L.off_bins);
  d.scan_tmp = (uint64_t*)(w + L.off_scan);
  d.counters = (uint64_t*)(w + L.off_cnt);
  d.aside = (uint64_t*)(w + L.off_aside);
  c->snap = (uint64_t*)(w + L.off_snap);
  d.shadow = (int8_t*)(w + L.off_shadow);
  c->flag_dev = (int*)(w + L.off_flag);
  d.bk_cnt = (uint32_t*)(w + L.off_bkc);
  d.bk_off = (uint64_t*)(w + L.off_bko);
  const bool staged = stage_possible(&c->prm);
  d.stg_ent = staged ? (uint64_t*)(w + L.off_stg_ent) : nullptr;
  d.stg_cur = staged ? (unsigned long long*)(w + L.off_stg_cur) : nullptr;
  const bool gram = gram_possible(&c->prm);
  d.cls_nodes = gram || staged ? (int32_t*)(w + L.off_cls_nodes) : nullptr;
  d.cls_count = gram || staged ? (uint32_t*)(w + L.off_cls_count) : nullptr;
}

// Fill in a default-constructed context (no allocation of any kind): layout,
// cleared counters, per-vector norms, int8 copy.  `may_sync` = the caller allows
// a stream synchronisation: float32 data qualify for the matrix-core join only
// after a device-side check whose verdict has to be read back; without it float
// data take the general join (uint8 data always qualify, nothing is read back).
int init_ctx(gnnd_ctx* c, const gnnd_params* prm, const Layout& L, const void* vec_a,
             const void* vec_b, int64_t split, bool merge_mode, bool may_sync) {
  c->prm = *prm;
  c->stream = (hipStream_t)prm->stream;
  c->sh = Shape{prm->n, prm->d, prm->k, prm->p, prm->metric, split, vec_a, vec_b,
                prm->update_mode == GNND_UPDATE_ALL_PAIRS ? 1 : 0};
  // one segment of 32 is the plain list
  c->sh.segments = prm->list_mode == GNND_LISTS_SEGMENTED ? prm->k / 32 : 1;
  c->iter = 0;
  c->stage = 0;
  c->has_graph = false;
  c->fresh_random = false;
  c->merge_mode = merge_mode;
  c->have_events = false;
  c->prof_on = false;
  c->prof_count = 0;
  c->prof_missed = 0;
  bind(c, L);
  // the statistics counters start at zero; the slot words read "nothing received" until the
  // first sampling stage writes them
  hipError_t e = launch_zero_u32((uint32_t*)c->ds.pslot, 2 * (size_t)prm->n, c->stream);
  if (e == hipSuccess)
    e = launch_zero_u32((uint32_t*)c->ds.counters, (size_t)kStripes * C_SLOTS * 2, c->stream);
  if (e != hipSuccess) return hip_fail(nullptr, e, "clearing workspace counters");
  if (needs_norms(prm)) {  // the cosine distance divides by them, the float32 matrix-core
                           // join turns inner products into distances with them
    float* norms = reinterpret_cast<float*>(static_cast<char*>(prm->workspace_dev) + L.off_norms);
    c->sh.norms = norms;
    e = launch_row_norms(c->sh, norms, c->stream);
    if (e != hipSuccess) return hip_fail(nullptr, e, "row norm kernel");
  }
  // matrix-core path: build the int8 copy; float data qualifies only when every
  // value is an integer in 0..255 (then all distances are exact either way)
  c->use_mfma = false;
  if (mfma_possible(prm) && (may_sync || prm->metric == GNND_L2SQ_U8)) {
    int bad = 0;
    e = launch_zero_u32((uint32_t*)c->flag_dev, 1, c->stream);
    if (e == hipSuccess) e = launch_pack_i8(c->sh, c->ds, c->flag_dev, c->stream);
    if (prm->metric != GNND_L2SQ_U8) {  // bytes always fit; floats have to be looked at
      if (e == hipSuccess)
        e = hipMemcpyAsync(&bad, c->flag_dev, sizeof bad, hipMemcpyDeviceToHost, c->stream);
      if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    }
    if (e != hipSuccess) return hip_fail(nullptr, e, "packing vectors to int8");
    c->use_mfma = (bad == 0);
  }
  c->use_gram = gram_possible(prm) && !c->use_mfma;
  if (c->use_gram) {
    e = launch_gram_norms(c->sh, c->ds, c->stream);
    if (e != hipSuccess) return hip_fail(nullptr, e, "row norm kernel");
  }
  if ((prm->join_path == GNND_JOIN_MFMA || prm->join_path == GNND_JOIN_MFMA_DIRECT) && !c->use_mfma)
    return fail(nullptr, GNND_EINVAL,
                may_sync ? "GNND_JOIN_MFMA needs d <= 128, p <= 32 and uint8 vectors or float32 vectors "
                           "holding integers 0..255 with the squared-L2 metric"
                         : "GNND_JOIN_MFMA needs d <= 128, p <= 32 and uint8 vectors here (float32 "
                           "vectors have to be checked, which synchronises: use gnnd_create)");
  return GNND_OK;
}

const char* check_pointers(const gnnd_params* prm, const void* vec_a, const void* vec_b) {
  if (!vec_a) return "vectors pointer is NULL";
  if (((uintptr_t)vec_a & 15) || ((uintptr_t)vec_b & 15)) return "vectors must be 16-byte aligned";
  if (!prm->workspace_dev) return "workspace is NULL";
  if ((uintptr_t)prm->workspace_dev & 255) return "workspace must be 256-byte aligned";
  return nullptr;
}

// Shared by gnnd_create and gnnd_merge.
int create_impl(gnnd_ctx** out, const gnnd_params* prm, const void* vec_a, const void* vec_b,
                int64_t split, bool merge_mode) {
  if (!out) return fail(nullptr, GNND_EINVAL, "out is NULL");
  *out = nullptr;
  if (const char* m = check_params(prm)) return fail(nullptr, GNND_EINVAL, m);
  if (const char* m = check_pointers(prm, vec_a, vec_b)) return fail(nullptr, GNND_EINVAL, m);
  Layout L = make_layout(prm, merge_mode);
  if (prm->workspace_bytes < L.total) {
    char buf[128];
    snprintf(buf, sizeof buf, "workspace too small: %zu bytes given, %zu needed",
             prm->workspace_bytes, L.total);
    return fail(nullptr, GNND_ENOSPC, buf);
  }
  gnnd_ctx* c = new (std::nothrow) gnnd_ctx();
  if (!c) return fail(nullptr, GNND_EINVAL, "out of host memory");
  const int rc = init_ctx(c, prm, L, vec_a, vec_b, split, merge_mode, true);
  if (rc != GNND_OK) {
    delete c;
    return rc;
  }
  *out = c;
  return GNND_OK;
}

int ensure_events(gnnd_ctx* c) {
  if (c->have_events) return GNND_OK;
  for (int i = 0; i < kProfEvents; ++i) {
    hipError_t e = hipEventCreate(&c->ev[i]);
    if (e != hipSuccess) return hip_fail(c, e, "hipEventCreate");
  }
  c->have_events = true;
  return GNND_OK;
}

int read_stats(gnnd_ctx* c, gnnd_iter_stats* out) {
  constexpr int N = kStripes * C_SLOTS;
  uint64_t host[2 * N];
  hipError_t e = hipMemcpyAsync(host, c->ds.counters, N * 8, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(host + N, c->snap, N * 8, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hip_fail(c, e, "reading counters");
  uint64_t tot[C_SLOTS] = {0};
  for (int s = 0; s < kStripes; ++s)
    for (int j = 0; j < C_SLOTS; ++j) tot[j] += host[s * C_SLOTS + j] - host[N + s * C_SLOTS + j];
  memset(out, 0, sizeof *out);
  out->iter = c->iter;
  out->inserts = tot[C_INSERTS];
  out->dist_evals = tot[C_EVALS];
  out->sum_new = tot[C_SUMNEW];
  out->sum_old = tot[C_SUMOLD];
  out->proposals = tot[C_PROPS];
  out->dropped = tot[C_OVERFLOW];
  out->passed = tot[C_PASSED];
  return GNND_OK;
}

int step_sample(gnnd_ctx* c) {
  if (!c->has_graph) return fail(c, GNND_ESTATE, "no graph: call gnnd_init_random or gnnd_set_graph first");
  if (c->stage != 0) return fail(c, GNND_ESTATE, "stage order is sample, join, update");
  // the counters only grow: keep their values from before this iteration
  hipError_t e = launch_copy_u64(c->snap, c->ds.counters, (size_t)kStripes * C_SLOTS, c->stream);
  if (e != hipSuccess) return hip_fail(c, e, "counter snapshot");
  e = launch_sample(c->sh, c->ds, c->prm.seed, (uint32_t)(c->iter + 1), c->stream);
  if (e != hipSuccess) return hip_fail(c, e, "sampling kernels");
  c->stage = 1;
  return GNND_OK;
}
// `after_join` (may be NULL) is recorded behind the cross-matching kernel itself, in front of
// the pass that moves staged results into the destinations' segments (where there is one).
int step_join(gnnd_ctx* c, hipEvent_t after_join = nullptr) {
  if (c->stage != 1) return fail(c, GNND_ESTATE, "stage order is sample, join, update");
  hipError_t e;
  if (c->use_mfma) {
    e = launch_join_mfma(c->sh, c->ds, c->merge_mode, c->fresh_random, c->stream, after_join);
  } else {
    e = c->use_gram ? launch_join_gram(c->sh, c->ds, c->merge_mode, c->stream)
                    : launch_join(c->sh, c->ds, c->prm.join_path, c->merge_mode, c->stream);
    if (after_join) (void)hipEventRecord(after_join, c->stream);
  }
  if (e != hipSuccess) return hip_fail(c, e, "join kernel");
  c->stage = 2;
  return GNND_OK;
}
int step_update(gnnd_ctx* c) {
  if (c->stage != 2) return fail(c, GNND_ESTATE, "stage order is sample, join, update");
  hipError_t e = launch_update(c->sh, c->ds, c->stream);
  if (e != hipSuccess) return hip_fail(c, e, "update kernels");
  c->stage = 0;
  c->iter += 1;
  c->fresh_random = false;
  return GNND_OK;
}

int iterate_impl(gnnd_ctx* c, gnnd_iter_stats* out) {
  int rc;
  if (!out && c->prof_on && (size_t)c->prof_count * kProfEvents >= c->prof.size())
    c->prof_missed += 1;
  if (!out && c->prof_on && (size_t)c->prof_count * kProfEvents < c->prof.size()) {
    hipEvent_t* ev = &c->prof[(size_t)c->prof_count * kProfEvents];
    (void)hipEventRecord(ev[0], c->stream);
    if ((rc = step_sample(c)) != GNND_OK) return rc;
    (void)hipEventRecord(ev[1], c->stream);
    if ((rc = step_join(c, ev[2])) != GNND_OK) return rc;
    (void)hipEventRecord(ev[3], c->stream);
    if ((rc = step_update(c)) != GNND_OK) return rc;
    (void)hipEventRecord(ev[4], c->stream);
    c->prof_count += 1;
    return GNND_OK;
  }
  if (out) {
    if ((rc = ensure_events(c)) != GNND_OK) return rc;
    (void)hipEventRecord(c->ev[0], c->stream);
  }
  if ((rc = step_sample(c)) != GNND_OK) return rc;
  if (out) (void)hipEventRecord(c->ev[1], c->stream);
  if ((rc = step_join(c, out ? c->ev[2] : nullptr)) != GNND_OK) return rc;
  if (out) (void)hipEventRecord(c->ev[3], c->stream);
  if ((rc = step_update(c)) != GNND_OK) return rc;
  if (out) {
    (void)hipEventRecord(c->ev[4], c->stream);
    if ((rc = read_stats(c, out)) != GNND_OK) return rc;
    (void)hipEventElapsedTime(&out->ms_sample, c->ev[0], c->ev[1]);
    (void)hipEventElapsedTime(&out->ms_join, c->ev[1], c->ev[2]);
    (void)hipEventElapsedTime(&out->ms_handout, c->ev[2], c->ev[3]);
    (void)hipEventElapsedTime(&out->ms_update, c->ev[3], c->ev[4]);
  }
  return GNND_OK;
}

// ---------------------------------------------------------------------------
// GGM on two sets given in collection ids (shared by gnnd_merge and the shard driver).
int merge_impl(const gnnd_params* prm, const void* vec1, int64_t n1, int64_t base1,
               const void* vec2, int64_t n2, int64_t base2, int64_t id_space,
               const int32_t* ids1, const void* dist1, const int32_t* ids2, const void* dist2,
               int32_t iters, int32_t* ids_out, void* dist_out, gnnd_iter_stats* stats) {
  if (const char* m = check_params(prm)) return fail(nullptr, GNND_EINVAL, m);
  if (prm->list_mode != GNND_LISTS_PLAIN)
    return fail(nullptr, GNND_EINVAL, "the merge works on plain lists (list_mode 0)");
  if (n1 <= 0 || n2 <= 0 || n1 + n2 != prm->n)
    return fail(nullptr, GNND_EINVAL, "n1 + n2 must equal params.n, both positive");
  if (n1 <= prm->k || n2 <= prm->k)
    return fail(nullptr, GNND_EINVAL, "each input graph needs more than k nodes");
  if (base1 < 0 || base2 < 0 || base1 + n1 > id_space || base2 + n2 > id_space ||
      (base1 < base2 + n2 && base2 < base1 + n1))
    return fail(nullptr, GNND_EINVAL, "the two id ranges must be disjoint and inside id_space");
  if (prm->n + id_space > ((int64_t)1 << 30))
    return fail(nullptr, GNND_EINVAL, "n + id_space must be <= 2^30");
  if (iters < 0) return fail(nullptr, GNND_EINVAL, "iters must be >= 0");
  if (!vec2 || !ids1 || !dist1 || !ids2 || !dist2 || !ids_out || !dist_out)
    return fail(nullptr, GNND_EINVAL, "NULL pointer argument");
  gnnd_ctx* c = nullptr;
  int rc = create_impl(&c, prm, vec1, vec2, n1, true);
  if (rc != GNND_OK) return rc;
  const MergeIds mi{n1, base1, n2, base2};
  hipError_t e =
      c->use_mfma
          ? launch_merge_init_i8(c->sh, c->ds, prm->seed, mi, ids1, dist1, ids2, dist2, c->stream)
          : launch_merge_init(c->sh, c->ds, prm->seed, mi, ids1, dist1, ids2, dist2, c->stream);
  if (e != hipSuccess) {
    rc = hip_fail(nullptr, e, "merge init kernel");
  } else {
    c->has_graph = true;
    for (int32_t t = 0; t < iters && rc == GNND_OK; ++t)
      rc = iterate_impl(c, stats ? stats + t : nullptr);
    if (rc == GNND_OK) {
      e = launch_merge_final(c->sh, c->ds, mi, ids_out, dist_out, c->stream);
      if (e != hipSuccess) rc = hip_fail(nullptr, e, "merge final kernel");
    } else {
      g_last_error = c->err;
    }
  }
  gnnd_destroy(c);
  return rc;
}

// ---------------------------------------------------------------------------
// Out-of-core scheme of Sec. 5.1 on one GPU: equal shards of consecutive rows
// live in (pinned) host memory; each is built on its own, then every pair of
// shards is merged once and stored back as two sub-graphs.  Two device slots
// alternate, so a copy stream moves the next step's data in and the previous
// step's results out while the compute stream works.
struct ShardPlan {
  int shards;
  int64_t size, last, maxs;  // rows per shard, rows of the last shard, larger of the two
  size_t elem, vec_bytes, graph_bytes, off_vec[2][2], off_ids[2][2], off_dist[2][2],
      off_oids[2], off_odist[2], off_ws, ws_bytes, total;
};

const char* plan_shards(const gnnd_params* prm, int32_t shards, ShardPlan* pl) {
  if (!prm) return "params is NULL";
  if (prm->list_mode != GNND_LISTS_PLAIN) return "the shard driver works on plain lists (list_mode 0)";
  if (shards < 2 || shards > 1024) return "shards must be in [2, 1024]";
  gnnd_params q = *prm;
  pl->shards = shards;
  pl->size = prm->n / shards;
  pl->last = prm->n - pl->size * (shards - 1);
  pl->maxs = pl->last > pl->size ? pl->last : pl->size;
  if (pl->size <= prm->k) return "every shard needs more than k rows";
  q.n = pl->size + pl->maxs;  // the largest merge
  if (const char* m = check_params(&q)) return m;
  if (q.n + prm->n > ((int64_t)1 << 30)) return "collection too large: 2 shards + n must be <= 2^30";
  pl->elem = prm->metric == GNND_L2SQ_U8 ? 1 : 4;
  pl->vec_bytes = (size_t)pl->maxs * prm->d * pl->elem;
  pl->graph_bytes = (size_t)pl->maxs * prm->k * 4;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  for (int s = 0; s < 2; ++s) {
    for (int h = 0; h < 2; ++h) {
      pl->off_vec[s][h] = take(pl->vec_bytes);
      pl->off_ids[s][h] = take(pl->graph_bytes);
      pl->off_dist[s][h] = take(pl->graph_bytes);
    }
    pl->off_oids[s] = take(2 * pl->graph_bytes);
    pl->off_odist[s] = take(2 * pl->graph_bytes);
  }
  pl->ws_bytes = make_layout(&q, true).total;
  pl->off_ws = take(pl->ws_bytes);
  pl->total = o;
  return nullptr;
}

// Every unordered pair of 0..S-1 exactly once, as rounds of disjoint pairs
// (circle method): consecutive merges mostly touch different shards.
std::vector<std::pair<int, int>> pair_schedule(int S) {
  std::vector<std::pair<int, int>> out;
  const int m = (S % 2) ? S + 1 : S;  // odd: one bye per round
  for (int r = 0; r < m - 1; ++r)
    for (int i = 0; i < m / 2; ++i) {
      int a = i == 0 ? m - 1 : (r + i) % (m - 1);
      int b = i == 0 ? r : (r - i + (m - 1)) % (m - 1);
      if (a >= S || b >= S) continue;
      out.emplace_back(a < b ? a : b, a < b ? b : a);
    }
  return out;
}

#define GNND_HIP(call, what)                        \
  do {                                              \
    hipError_t e_ = (call);                         \
    if (e_ != hipSuccess) { rc = hip_fail(nullptr, e_, what); goto done; } \
  } while (0)

// Where the collection and its graph live while they are not on the GPU:
// pinned host arrays, or three files behind one pinned staging buffer.  In file
// mode every transfer is cut into pieces of half the staging buffer; a piece is
// read (or written) by a host function on a stream of the store's own while the
// copy stream moves the other half over the bus, so file access, bus transfers
// and the compute stream's kernels all overlap (Sec. 5.1: reading and writing
// the sub-graphs takes place while the GPU works).  All file accesses run in the
// order they were enqueued, so a sub-graph is read back only after it has been
// written.  A failed read leaves zeros in the buffer (valid ids and distances)
// and is reported when the call ends.
struct ShardStore {
  enum Which { kVec = 0, kIds = 1, kDist = 2 };
  char* mem[3] = {nullptr, nullptr, nullptr};
  int fd[3] = {-1, -1, -1};
  char* staging = nullptr;
  size_t half = 0;                  // bytes per half of the staging buffer
  hipStream_t io = nullptr;         // runs the host functions that touch the files
  hipEvent_t filled[2] = {nullptr, nullptr};   // a half holds a piece ready to leave
  hipEvent_t drained[2] = {nullptr, nullptr};  // a half's piece has left (copied or written)
  unsigned piece = 0;
  std::atomic<int> io_errno{0};
  struct Job { ShardStore* st; int fd; bool write; char* buf; size_t bytes; off_t at; };
  std::deque<Job> jobs;  // stable addresses until the streams have drained

  bool files() const { return staging != nullptr; }
  hipError_t open_streams() {
    hipError_t e = hipStreamCreateWithFlags(&io, hipStreamNonBlocking);
    for (int i = 0; i < 2 && e == hipSuccess; ++i) {
      e = hipEventCreateWithFlags(&filled[i], hipEventDisableTiming);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&drained[i], hipEventDisableTiming);
    }
    return e;
  }
  hipError_t drain() { return io ? hipStreamSynchronize(io) : hipSuccess; }
  ~ShardStore() {
    if (io) {
      (void)hipStreamSynchronize(io);
      (void)hipStreamDestroy(io);
    }
    for (int i = 0; i < 2; ++i) {
      if (filled[i]) (void)hipEventDestroy(filled[i]);
      if (drained[i]) (void)hipEventDestroy(drained[i]);
    }
    for (int i = 0; i < 3; ++i)
      if (fd[i] >= 0) ::close(fd[i]);
  }
  // one contiguous range of a piece, read or written to the end
  static void transfer(Job* j, size_t from, size_t to) {
    size_t done = from;
    while (done < to) {
      const ssize_t r = j->write ? ::pwrite(j->fd, j->buf + done, to - done, j->at + (off_t)done)
                                 : ::pread(j->fd, j->buf + done, to - done, j->at + (off_t)done);
      if (r > 0) { done += (size_t)r; continue; }
      if (r < 0 && errno == EINTR) continue;
      int expected = 0;
      j->st->io_errno.compare_exchange_strong(expected, r < 0 ? errno : EIO);
      if (!j->write) memset(j->buf + done, 0, to - done);
      break;
    }
  }
  // a piece: large ones are split over a few threads (one thread copies from
  // the page cache at a fraction of what the bus moves)
  static void run(void* arg) {
    Job* j = static_cast<Job*>(arg);
    constexpr size_t kPerThread = (size_t)8 << 20;
    constexpr int kMaxThreads = 4;
    int parts = (int)(j->bytes / kPerThread);
    parts = parts < 1 ? 1 : (parts > kMaxThreads ? kMaxThreads : parts);
    const size_t step = ((j->bytes + parts - 1) / parts + 4095) & ~(size_t)4095;
    std::thread helpers[kMaxThreads - 1];
    int started = 0;
    for (int t = 1; t < parts; ++t) {
      const size_t from = (size_t)t * step, to = from + step < j->bytes ? from + step : j->bytes;
      if (from >= to) break;
      try {
        helpers[started] = std::thread(transfer, j, from, to);
        ++started;
      } catch (...) {
        transfer(j, from, to);  // no thread to be had: do it here
      }
    }
    transfer(j, 0, step < j->bytes ? step : j->bytes);
    for (int t = 0; t < started; ++t) helpers[t].join();
  }
  hipError_t up(hipStream_t copy, void* dev, int which, size_t at, size_t bytes) {
    if (!files()) return hipMemcpyAsync(dev, mem[which] + at, bytes, hipMemcpyHostToDevice, copy);
    for (size_t o = 0; o < bytes; o += half) {
      const size_t len = bytes - o < half ? bytes - o : half;
      const int h = (int)(piece++ & 1);
      char* buf = staging + (size_t)h * half;
      hipError_t e = hipStreamWaitEvent(io, drained[h], 0);
      if (e != hipSuccess) return e;
      jobs.push_back(Job{this, fd[which], false, buf, len, (off_t)(at + o)});
      if ((e = hipLaunchHostFunc(io, &ShardStore::run, &jobs.back())) != hipSuccess) return e;
      if ((e = hipEventRecord(filled[h], io)) != hipSuccess) return e;
      if ((e = hipStreamWaitEvent(copy, filled[h], 0)) != hipSuccess) return e;
      e = hipMemcpyAsync((char*)dev + o, buf, len, hipMemcpyHostToDevice, copy);
      if (e != hipSuccess) return e;
      if ((e = hipEventRecord(drained[h], copy)) != hipSuccess) return e;
    }
    return hipSuccess;
  }
  hipError_t down(hipStream_t copy, int which, size_t at, const void* dev, size_t bytes) {
    if (!files()) return hipMemcpyAsync(mem[which] + at, dev, bytes, hipMemcpyDeviceToHost, copy);
    for (size_t o = 0; o < bytes; o += half) {
      const size_t len = bytes - o < half ? bytes - o : half;
      const int h = (int)(piece++ & 1);
      char* buf = staging + (size_t)h * half;
      hipError_t e = hipStreamWaitEvent(copy, drained[h], 0);
      if (e != hipSuccess) return e;
      e = hipMemcpyAsync(buf, (const char*)dev + o, len, hipMemcpyDeviceToHost, copy);
      if (e != hipSuccess) return e;
      if ((e = hipEventRecord(filled[h], copy)) != hipSuccess) return e;
      if ((e = hipStreamWaitEvent(io, filled[h], 0)) != hipSuccess) return e;
      jobs.push_back(Job{this, fd[which], true, buf, len, (off_t)(at + o)});
      if ((e = hipLaunchHostFunc(io, &ShardStore::run, &jobs.back())) != hipSuccess) return e;
      if ((e = hipEventRecord(drained[h], io)) != hipSuccess) return e;
    }
    return hipSuccess;
  }
};

int run_sharded(const gnnd_params* prm, const ShardPlan& pl, ShardStore& store,
                int32_t build_iters, int32_t merge_iters, hipStream_t copy,
                gnnd_shard_stats* stats) {
  int rc = GNND_OK;
  char* arena = (char*)prm->workspace_dev;
  hipStream_t comp = (hipStream_t)prm->stream;
  const int k = prm->k;
  const size_t row_vec = (size_t)prm->d * pl.elem, row_g = (size_t)k * 4;
  auto base_of = [&](int s) { return (int64_t)s * pl.size; };
  auto rows_of = [&](int s) { return s == pl.shards - 1 ? pl.last : pl.size; };
  hipEvent_t ev_up[2] = {nullptr, nullptr}, ev_done[2] = {nullptr, nullptr}, t0 = nullptr,
             t1 = nullptr, t2 = nullptr;
  const auto pairs = pair_schedule(pl.shards);
  const auto wall0 = std::chrono::steady_clock::now();
  for (int i = 0; i < 2; ++i) {
    GNND_HIP(hipEventCreateWithFlags(&ev_up[i], hipEventDisableTiming), "hipEventCreate");
    GNND_HIP(hipEventCreateWithFlags(&ev_done[i], hipEventDisableTiming), "hipEventCreate");
  }
  GNND_HIP(hipEventCreate(&t0), "hipEventCreate");
  GNND_HIP(hipEventCreate(&t1), "hipEventCreate");
  GNND_HIP(hipEventCreate(&t2), "hipEventCreate");
  GNND_HIP(hipEventRecord(t0, comp), "hipEventRecord");

  // ---- phase 1: one graph per shard ------------------------------------------
  {
    auto upload = [&](int s) {  // vectors of shard s into slot s % 2
      return store.up(copy, arena + pl.off_vec[s % 2][0], ShardStore::kVec,
                      (size_t)base_of(s) * row_vec, (size_t)rows_of(s) * row_vec);
    };
    GNND_HIP(upload(0), "shard upload");
    GNND_HIP(hipEventRecord(ev_up[0], copy), "hipEventRecord");
    for (int s = 0; s < pl.shards; ++s) {
      const int slot = s % 2;
      if (s + 1 < pl.shards) {  // next shard's vectors travel while this one is built
        if (s >= 1) GNND_HIP(hipStreamWaitEvent(copy, ev_done[1 - slot], 0), "hipStreamWaitEvent");
        GNND_HIP(upload(s + 1), "shard upload");
        GNND_HIP(hipEventRecord(ev_up[1 - slot], copy), "hipEventRecord");
      }
      GNND_HIP(hipStreamWaitEvent(comp, ev_up[slot], 0), "hipStreamWaitEvent");
      gnnd_params q = *prm;
      q.n = rows_of(s);
      q.seed = prm->seed + (uint64_t)s;
      q.workspace_dev = arena + pl.off_ws;
      q.workspace_bytes = pl.ws_bytes;
      gnnd_ctx* c = nullptr;
      rc = create_impl(&c, &q, arena + pl.off_vec[slot][0], nullptr, q.n, false);
      if (rc != GNND_OK) goto done;
      rc = gnnd_build(c, build_iters, 0.f, nullptr);
      if (rc == GNND_OK) {
        hipError_t e = launch_get_graph(c->sh, c->ds, (int32_t*)(arena + pl.off_oids[slot]),
                                        arena + pl.off_odist[slot], nullptr,
                                        (int32_t)base_of(s), comp);
        if (e != hipSuccess) rc = hip_fail(nullptr, e, "get_graph kernel");
      } else {
        g_last_error = c->err;
      }
      gnnd_destroy(c);
      if (rc != GNND_OK) goto done;
      GNND_HIP(hipEventRecord(ev_done[slot], comp), "hipEventRecord");
      GNND_HIP(hipStreamWaitEvent(copy, ev_done[slot], 0), "hipStreamWaitEvent");
      GNND_HIP(store.down(copy, ShardStore::kIds, (size_t)base_of(s) * row_g,
                          arena + pl.off_oids[slot], (size_t)rows_of(s) * row_g), "graph download");
      GNND_HIP(store.down(copy, ShardStore::kDist, (size_t)base_of(s) * row_g,
                          arena + pl.off_odist[slot], (size_t)rows_of(s) * row_g), "graph download");
    }
  }
  GNND_HIP(hipEventRecord(t1, comp), "hipEventRecord");

  // ---- phase 2: every pair of shards merged once -------------------------------
  {
    // what of merge m can travel before merge m-1 has delivered: the vectors, and the
    // graph of a shard that merge m-1 does not touch
    auto up_vec = [&](int m) {
      const int slot = m % 2;
      const int sh[2] = {pairs[m].first, pairs[m].second};
      for (int h = 0; h < 2; ++h) {
        hipError_t e = store.up(copy, arena + pl.off_vec[slot][h], ShardStore::kVec,
                                (size_t)base_of(sh[h]) * row_vec, (size_t)rows_of(sh[h]) * row_vec);
        if (e != hipSuccess) return e;
      }
      return hipSuccess;
    };
    auto up_graph = [&](int m, int h) {
      const int slot = m % 2;
      const int s = h ? pairs[m].second : pairs[m].first;
      hipError_t e = store.up(copy, arena + pl.off_ids[slot][h], ShardStore::kIds,
                              (size_t)base_of(s) * row_g, (size_t)rows_of(s) * row_g);
      if (e != hipSuccess) return e;
      return store.up(copy, arena + pl.off_dist[slot][h], ShardStore::kDist,
                      (size_t)base_of(s) * row_g, (size_t)rows_of(s) * row_g);
    };
    auto touches = [&](int m, int s) { return pairs[m].first == s || pairs[m].second == s; };
    const int M = (int)pairs.size();
    // merge 0: everything is on the host already (the downloads above are earlier in `copy`)
    GNND_HIP(up_vec(0), "merge upload");
    GNND_HIP(up_graph(0, 0), "merge upload");
    GNND_HIP(up_graph(0, 1), "merge upload");
    GNND_HIP(hipEventRecord(ev_up[0], copy), "hipEventRecord");
    for (int m = 0; m < M; ++m) {
      const int slot = m % 2;
      const int sa = pairs[m].first, sb = pairs[m].second;
      bool late[2] = {false, false};
      if (m + 1 < M) {
        // slot 1-slot was last read by merge m-1 and its results were fetched after
        // ev_done[1-slot]; both are earlier in `copy` than what follows
        GNND_HIP(up_vec(m + 1), "merge upload");
        for (int h = 0; h < 2; ++h) {
          const int s = h ? pairs[m + 1].second : pairs[m + 1].first;
          late[h] = touches(m, s);
          if (!late[h]) GNND_HIP(up_graph(m + 1, h), "merge upload");
        }
      }
      GNND_HIP(hipStreamWaitEvent(comp, ev_up[slot], 0), "hipStreamWaitEvent");
      gnnd_params q = *prm;
      q.n = rows_of(sa) + rows_of(sb);
      q.seed = prm->seed + 1000 + (uint64_t)m;
      q.workspace_dev = arena + pl.off_ws;
      q.workspace_bytes = pl.ws_bytes;
      rc = merge_impl(&q, arena + pl.off_vec[slot][0], rows_of(sa), base_of(sa),
                      arena + pl.off_vec[slot][1], rows_of(sb), base_of(sb), prm->n,
                      (const int32_t*)(arena + pl.off_ids[slot][0]), arena + pl.off_dist[slot][0],
                      (const int32_t*)(arena + pl.off_ids[slot][1]), arena + pl.off_dist[slot][1],
                      merge_iters, (int32_t*)(arena + pl.off_oids[slot]),
                      arena + pl.off_odist[slot], nullptr);
      if (rc != GNND_OK) goto done;
      GNND_HIP(hipEventRecord(ev_done[slot], comp), "hipEventRecord");
      GNND_HIP(hipStreamWaitEvent(copy, ev_done[slot], 0), "hipStreamWaitEvent");
      // results: rows of shard sa, then rows of shard sb
      const size_t na = (size_t)rows_of(sa), nb = (size_t)rows_of(sb);
      GNND_HIP(store.down(copy, ShardStore::kIds, (size_t)base_of(sa) * row_g,
                          arena + pl.off_oids[slot], na * row_g), "merge download");
      GNND_HIP(store.down(copy, ShardStore::kIds, (size_t)base_of(sb) * row_g,
                          arena + pl.off_oids[slot] + na * row_g, nb * row_g), "merge download");
      GNND_HIP(store.down(copy, ShardStore::kDist, (size_t)base_of(sa) * row_g,
                          arena + pl.off_odist[slot], na * row_g), "merge download");
      GNND_HIP(store.down(copy, ShardStore::kDist, (size_t)base_of(sb) * row_g,
                          arena + pl.off_odist[slot] + na * row_g, nb * row_g), "merge download");
      if (m + 1 < M) {
        for (int h = 0; h < 2; ++h)
          if (late[h]) GNND_HIP(up_graph(m + 1, h), "merge upload");
        GNND_HIP(hipEventRecord(ev_up[1 - slot], copy), "hipEventRecord");
      }
    }
  }
  GNND_HIP(hipEventRecord(t2, comp), "hipEventRecord");
  GNND_HIP(hipStreamSynchronize(copy), "hipStreamSynchronize");
  GNND_HIP(hipStreamSynchronize(comp), "hipStreamSynchronize");
  GNND_HIP(store.drain(), "hipStreamSynchronize");
  if (stats) {
    memset(stats, 0, sizeof *stats);
    stats->builds = pl.shards;
    stats->merges = (int32_t)pairs.size();
    (void)hipEventElapsedTime(&stats->ms_build, t0, t1);
    (void)hipEventElapsedTime(&stats->ms_merge, t1, t2);
    stats->ms_total = std::chrono::duration<float, std::milli>(
                          std::chrono::steady_clock::now() - wall0).count();
  }
  if (const int err = store.io_errno.load())
    rc = fail(nullptr, GNND_EIO, (std::string("file access failed: ") + strerror(err)).c_str());
done:
  if (rc != GNND_OK && rc != GNND_EIO) {  // nothing enqueued may outlive the store
    (void)hipStreamSynchronize(copy);
    (void)hipStreamSynchronize(comp);
    (void)store.drain();
  }
  for (int i = 0; i < 2; ++i) {
    if (ev_up[i]) (void)hipEventDestroy(ev_up[i]);
    if (ev_done[i]) (void)hipEventDestroy(ev_done[i]);
  }
  if (t0) (void)hipEventDestroy(t0);
  if (t1) (void)hipEventDestroy(t1);
  if (t2) (void)hipEventDestroy(t2);
  return rc;
}
#undef GNND_HIP

// Device address of the static scratch array on the current device, looked up
// once per device (every GPU holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

int static_scratch_of(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, GNND_EINVAL, "device number out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetSymbolAddress(scratch)");
    if (!ptr || ((uintptr_t)ptr & 255))
      return fail(nullptr, GNND_EHIP, "the static scratch array has no usable device address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return GNND_OK;
}

}  // namespace

extern "C" {

size_t gnnd_workspace_bytes(const gnnd_params* prm) {
  if (check_params(prm)) return 0;
  return make_layout(prm, true).total;
}

int gnnd_create(gnnd_ctx** out, const gnnd_params* prm, const void* vectors_dev) {
  return create_impl(out, prm, vectors_dev, nullptr, prm ? prm->n : 0, false);
}

void gnnd_destroy(gnnd_ctx* c) {
  if (!c) return;
  if (c->have_events)
    for (int i = 0; i < kProfEvents; ++i) (void)hipEventDestroy(c->ev[i]);
  for (hipEvent_t ev : c->prof) (void)hipEventDestroy(ev);
  delete c;
}

const char* gnnd_last_error(const gnnd_ctx* c) { return c ? c->err.c_str() : g_last_error.c_str(); }

int gnnd_join_path(const gnnd_ctx* c) {
  if (!c) return GNND_EINVAL;
  return c->use_mfma ? GNND_JOIN_MFMA : c->use_gram ? GNND_JOIN_GRAM : GNND_JOIN_VALU;
}

int gnnd_set_profiling(gnnd_ctx* c, int iterations) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  if (iterations < 0 || iterations > kProfItersMax)
    return fail(c, GNND_EINVAL, "profiling window must be 0 (off) .. 65536 iterations");
  if (iterations > 0) {
    // the events are created here, outside any timed loop; a window never shrinks
    const size_t want =
        kProfEvents * (size_t)(iterations < kProfItersDefault ? kProfItersDefault : iterations);
    try {
      c->prof.reserve(want);
    } catch (...) {
      return fail(c, GNND_EINVAL, "out of host memory");
    }
    while (c->prof.size() < want) {
      hipEvent_t ev;
      hipError_t e = hipEventCreate(&ev);
      if (e != hipSuccess) return hip_fail(c, e, "hipEventCreate");
      c->prof.push_back(ev);
    }
  }
  c->prof_on = iterations != 0;
  c->prof_count = 0;
  c->prof_missed = 0;
  return GNND_OK;
}

int gnnd_get_stage_ms(gnnd_ctx* c, int32_t* count, int32_t* missed, float* ms_sample,
                      float* ms_join, float* ms_handout, float* ms_update) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  if (!count || !missed || !ms_sample || !ms_join || !ms_handout || !ms_update)
    return fail(c, GNND_EINVAL, "NULL output pointer");
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
  *count = c->prof_count;
  *missed = c->prof_missed;
  *ms_sample = *ms_join = *ms_handout = *ms_update = 0.f;
  for (int t = 0; t < c->prof_count; ++t) {
    const hipEvent_t* ev = &c->prof[(size_t)t * kProfEvents];
    float a = 0, b = 0, h = 0, d = 0;
    (void)hipEventElapsedTime(&a, ev[0], ev[1]);
    (void)hipEventElapsedTime(&b, ev[1], ev[2]);
    (void)hipEventElapsedTime(&h, ev[2], ev[3]);
    (void)hipEventElapsedTime(&d, ev[3], ev[4]);
    *ms_sample += a;
    *ms_join += b;
    *ms_handout += h;
    *ms_update += d;
  }
  c->prof_count = 0;
  c->prof_missed = 0;
  return GNND_OK;
}

int gnnd_init_random(gnnd_ctx* c) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  if (c->merge_mode) return fail(c, GNND_ESTATE, "context belongs to a merge");
  hipError_t e = c->use_mfma ? launch_init_random_i8(c->sh, c->ds, c->prm.seed, c->stream)
                             : launch_init_random(c->sh, c->ds, c->prm.seed, c->stream);
  if (e != hipSuccess) return hip_fail(c, e, "init kernel");
  c->has_graph = true;
  c->fresh_random = true;
  c->iter = 0;
  c->stage = 0;
  return GNND_OK;
}

int gnnd_iterate(gnnd_ctx* c, gnnd_iter_stats* out) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  return iterate_impl(c, out);
}

int gnnd_step_sample(gnnd_ctx* c) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  return step_sample(c);
}
int gnnd_step_join(gnnd_ctx* c) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  return step_join(c);
}
int gnnd_step_update(gnnd_ctx* c, gnnd_iter_stats* out) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  int rc = step_update(c);
  if (rc != GNND_OK) return rc;
  return out ? read_stats(c, out) : GNND_OK;
}

int gnnd_build(gnnd_ctx* c, int32_t max_iters, float delta, gnnd_iter_stats* last) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  if (max_iters < 0) return fail(c, GNND_EINVAL, "max_iters must be >= 0");
  if (!(delta >= 0.f)) return fail(c, GNND_EINVAL, "delta must be >= 0");
  int rc = gnnd_init_random(c);
  if (rc != GNND_OK) return rc;
  gnnd_iter_stats st;
  memset(&st, 0, sizeof st);
  for (int32_t t = 0; t < max_iters; ++t) {
    const bool want = delta > 0.f || (last && t == max_iters - 1);
    rc = iterate_impl(c, want ? &st : nullptr);
    if (rc != GNND_OK) return rc;
    if (delta > 0.f && (double)st.inserts < (double)delta * (double)c->prm.n * c->prm.k) break;
  }
  if (last) *last = st;
  return GNND_OK;
}

int gnnd_get_graph(gnnd_ctx* c, int32_t* ids, void* dist, uint8_t* isnew) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  if (!c->has_graph) return fail(c, GNND_ESTATE, "no graph yet");
  hipError_t e = launch_get_graph(c->sh, c->ds, ids, dist, isnew, 0, c->stream);
  return e == hipSuccess ? GNND_OK : hip_fail(c, e, "get_graph kernel");
}

int gnnd_set_graph(gnnd_ctx* c, const int32_t* ids, const void* dist, const uint8_t* isnew,
                   int32_t iter) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  if (!ids || !dist) return fail(c, GNND_EINVAL, "ids and dist are required");
  if (iter < 0) return fail(c, GNND_EINVAL, "iter must be >= 0");
  if (c->merge_mode) return fail(c, GNND_ESTATE, "context belongs to a merge");
  if (c->sh.segments > 1)
    return fail(c, GNND_ESTATE, "a graph cannot be loaded into segmented lists");
  // ids are checked on the device (they become row numbers); the verdict is fetched here
  int bad = 0;
  hipError_t e = launch_zero_u32((uint32_t*)c->flag_dev, 1, c->stream);
  if (e == hipSuccess) e = launch_set_graph(c->sh, c->ds, ids, dist, isnew, c->flag_dev, c->stream);
  if (e == hipSuccess)
    e = hipMemcpyAsync(&bad, c->flag_dev, sizeof bad, hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hip_fail(c, e, "set_graph kernel");
  if (bad) {
    c->has_graph = false;
    return fail(c, GNND_EINVAL, "graph holds ids outside 0..n-1 or a node in its own list");
  }
  c->has_graph = true;
  c->fresh_random = false;
  c->iter = iter;
  c->stage = 0;
  return GNND_OK;
}

int gnnd_get_samples(gnnd_ctx* c, int32_t* snew, int32_t* cnew, int32_t* sold, int32_t* cold) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  if (c->stage == 0 && c->iter == 0) return fail(c, GNND_ESTATE, "nothing sampled yet");
  const size_t n = (size_t)c->prm.n, L = 2 * (size_t)c->prm.p;
  hipError_t e = hipSuccess;
  if (snew) e = hipMemcpyAsync(snew, c->ds.snew, n * L * 4, hipMemcpyDeviceToDevice, c->stream);
  if (e == hipSuccess && sold)
    e = hipMemcpyAsync(sold, c->ds.sold, n * L * 4, hipMemcpyDeviceToDevice, c->stream);
  if (e == hipSuccess && cnew)
    e = hipMemcpyAsync(cnew, c->ds.cnew, n * 4, hipMemcpyDeviceToDevice, c->stream);
  if (e == hipSuccess && cold)
    e = hipMemcpyAsync(cold, c->ds.cold, n * 4, hipMemcpyDeviceToDevice, c->stream);
  return e == hipSuccess ? GNND_OK : hip_fail(c, e, "copying sample lists");
}

int gnnd_get_proposals(gnnd_ctx* c, int32_t* u, int32_t* v, void* dist) {
  if (!c) return fail(nullptr, GNND_EINVAL, "ctx is NULL");
  if (!u || !v || !dist) return fail(c, GNND_EINVAL, "u, v and dist are required");
  if (c->stage != 2) return fail(c, GNND_ESTATE, "proposals exist between join and update only");
  hipError_t e = launch_get_proposals(c->sh, c->ds, u, v, dist, c->stream);
  return e == hipSuccess ? GNND_OK : hip_fail(c, e, "get_proposals kernel");
}

int gnnd_merge(const gnnd_params* prm, const void* vec1, int64_t n1, int64_t base1,
               const void* vec2, int64_t n2, int64_t base2, int64_t id_space,
               const int32_t* ids1, const void* dist1, const int32_t* ids2, const void* dist2,
               int32_t iters, int32_t* ids_out, void* dist_out, gnnd_iter_stats* stats) {
  return merge_impl(prm, vec1, n1, base1, vec2, n2, base2, id_space, ids1, dist1, ids2, dist2,
                    iters, ids_out, dist_out, stats);
}

int gnnd_append(const gnnd_params* prm, const void* vec1, int64_t n1, const int32_t* ids1,
                const void* dist1, const void* vec2, int64_t n2, int32_t build_iters,
                int32_t merge_iters, int32_t* ids_out, void* dist_out) {
  if (const char* m = check_params(prm)) return fail(nullptr, GNND_EINVAL, m);
  if (n1 <= 0 || n2 <= 0 || n1 + n2 != prm->n)
    return fail(nullptr, GNND_EINVAL, "n1 + n2 must equal params.n, both positive");
  if (n1 <= prm->k || n2 <= prm->k)
    return fail(nullptr, GNND_EINVAL, "each set needs more than k objects");
  if (build_iters < 0 || merge_iters < 0)
    return fail(nullptr, GNND_EINVAL, "negative iteration count");
  if (!vec1 || !vec2 || !ids1 || !dist1 || !ids_out || !dist_out)
    return fail(nullptr, GNND_EINVAL, "NULL pointer argument");
  // sub-graph of the batch, written where the merge will read it: the last n2 rows of the output
  gnnd_params sub = *prm;
  sub.n = n2;
  sub.seed = prm->seed + 1;
  gnnd_ctx* c = nullptr;
  int rc = create_impl(&c, &sub, vec2, nullptr, n2, false);
  if (rc != GNND_OK) return rc;
  rc = gnnd_build(c, build_iters, 0.f, nullptr);
  int32_t* ids2 = ids_out + n1 * prm->k;
  void* dist2 = static_cast<char*>(dist_out) + (size_t)n1 * prm->k * 4;
  if (rc == GNND_OK) {
    hipError_t e = launch_get_graph(c->sh, c->ds, ids2, dist2, nullptr, (int32_t)n1, c->stream);
    if (e != hipSuccess) rc = hip_fail(nullptr, e, "get_graph kernel");
  } else {
    g_last_error = c->err;
  }
  gnnd_destroy(c);
  if (rc != GNND_OK) return rc;
  // the merge reads ids2/dist2 in its first kernel and writes the output in its last
  return merge_impl(prm, vec1, n1, 0, vec2, n2, n1, prm->n, ids1, dist1, ids2, dist2, merge_iters,
                    ids_out, dist_out, nullptr);
}

size_t gnnd_sharded_arena_bytes(const gnnd_params* prm, int32_t shards) {
  ShardPlan pl;
  if (plan_shards(prm, shards, &pl)) return 0;
  return pl.total;
}

int gnnd_build_sharded(const gnnd_params* prm, const void* vectors_host, int32_t shards,
                       int32_t build_iters, int32_t merge_iters, int32_t* ids_host,
                       void* dist_host, void* copy_stream, gnnd_shard_stats* stats) {
  ShardPlan pl;
  if (const char* m = plan_shards(prm, shards, &pl)) return fail(nullptr, GNND_EINVAL, m);
  if (!vectors_host || !ids_host || !dist_host)
    return fail(nullptr, GNND_EINVAL, "NULL pointer argument");
  if (build_iters < 0 || merge_iters < 0) return fail(nullptr, GNND_EINVAL, "negative iteration count");
  if (!prm->workspace_dev || ((uintptr_t)prm->workspace_dev & 255))
    return fail(nullptr, GNND_EINVAL, "arena must be a 256-byte aligned device pointer");
  if (prm->workspace_bytes < pl.total) return fail(nullptr, GNND_ENOSPC, "arena too small");
  if (!copy_stream || copy_stream == prm->stream)
    return fail(nullptr, GNND_EINVAL, "copy_stream must be a stream of its own");
  ShardStore store;
  store.mem[ShardStore::kVec] = (char*)const_cast<void*>(vectors_host);
  store.mem[ShardStore::kIds] = (char*)ids_host;
  store.mem[ShardStore::kDist] = (char*)dist_host;
  return run_sharded(prm, pl, store, build_iters, merge_iters, (hipStream_t)copy_stream, stats);
}

int gnnd_build_sharded_files(const gnnd_params* prm, const char* vectors_path, int32_t shards,
                             int32_t build_iters, int32_t merge_iters, const char* ids_path,
                             const char* dist_path, void* staging_host, size_t staging_bytes,
                             void* copy_stream, gnnd_shard_stats* stats) {
  ShardPlan pl;
  if (const char* m = plan_shards(prm, shards, &pl)) return fail(nullptr, GNND_EINVAL, m);
  if (!vectors_path || !ids_path || !dist_path || !staging_host)
    return fail(nullptr, GNND_EINVAL, "NULL pointer argument");
  if (build_iters < 0 || merge_iters < 0) return fail(nullptr, GNND_EINVAL, "negative iteration count");
  if (staging_bytes < ((size_t)1 << 20))
    return fail(nullptr, GNND_EINVAL, "staging buffer must hold at least 1 MiB");
  if (!prm->workspace_dev || ((uintptr_t)prm->workspace_dev & 255))
    return fail(nullptr, GNND_EINVAL, "arena must be a 256-byte aligned device pointer");
  if (prm->workspace_bytes < pl.total) return fail(nullptr, GNND_ENOSPC, "arena too small");
  if (!copy_stream || copy_stream == prm->stream)
    return fail(nullptr, GNND_EINVAL, "copy_stream must be a stream of its own");
  ShardStore store;
  store.staging = static_cast<char*>(staging_host);
  store.half = (staging_bytes / 2) & ~(size_t)4095;
  const size_t vec_total = (size_t)prm->n * prm->d * pl.elem, g_total = (size_t)prm->n * prm->k * 4;
  store.fd[ShardStore::kVec] = ::open(vectors_path, O_RDONLY);
  if (store.fd[ShardStore::kVec] < 0)
    return fail(nullptr, GNND_EIO, (std::string("cannot open ") + vectors_path + ": " +
                                    strerror(errno)).c_str());
  struct stat sb;
  if (::fstat(store.fd[ShardStore::kVec], &sb) != 0 || (size_t)sb.st_size < vec_total)
    return fail(nullptr, GNND_EIO, "the vector file is shorter than n*d elements");
  const char* out_path[2] = {ids_path, dist_path};
  for (int i = 0; i < 2; ++i) {
    const int fd = ::open(out_path[i], O_RDWR | O_CREAT, 0644);
    store.fd[ShardStore::kIds + i] = fd;
    if (fd < 0 || ::ftruncate(fd, (off_t)g_total) != 0)
      return fail(nullptr, GNND_EIO, (std::string("cannot create ") + out_path[i] + ": " +
                                      strerror(errno)).c_str());
  }
  if (hipError_t e = store.open_streams()) return hip_fail(nullptr, e, "creating the file stream");
  return run_sharded(prm, pl, store, build_iters, merge_iters, (hipStream_t)copy_stream, stats);
}

int gnnd_build_static(const gnnd_params* prm, const void* vectors_dev, int32_t max_iters,
                      int32_t* ids_out_dev, void* dist_out_dev) {
  if (const char* m = check_params(prm)) return fail(nullptr, GNND_EINVAL, m);
  if (max_iters < 0) return fail(nullptr, GNND_EINVAL, "max_iters must be >= 0");
  if (!ids_out_dev || !dist_out_dev) return fail(nullptr, GNND_EINVAL, "NULL output pointer");
  gnnd_params q = *prm;
  q.workspace_dev = nullptr;
  q.workspace_bytes = 0;
  const Layout L = make_layout(&q, false);
  if (L.total > kStaticScratchBytes) {
    char buf[192];
    snprintf(buf, sizeof buf,
             "these parameters need %zu bytes of scratch, the static array holds %zu: use "
             "gnnd_create / gnnd_build with a workspace of the caller's",
             L.total, kStaticScratchBytes);
    return fail(nullptr, GNND_ENOSPC, buf);
  }
  void* base = nullptr;
  if (int rc = static_scratch_of(&base)) return rc;
  q.workspace_dev = base;
  q.workspace_bytes = kStaticScratchBytes;
  if (const char* m = check_pointers(&q, vectors_dev, nullptr)) return fail(nullptr, GNND_EINVAL, m);
  gnnd_ctx c;  // on the stack: nothing is allocated on the host either
  int rc = init_ctx(&c, &q, L, vectors_dev, nullptr, q.n, false, /*may_sync=*/false);
  if (rc == GNND_OK) rc = gnnd_build(&c, max_iters, 0.f, nullptr);
  if (rc == GNND_OK) {
    hipError_t e = launch_get_graph(c.sh, c.ds, ids_out_dev, dist_out_dev, nullptr, 0, c.stream);
    if (e != hipSuccess) rc = hip_fail(nullptr, e, "get_graph kernel");
  } else if (!c.err.empty()) {
    g_last_error = c.err;
  }
  return rc;
}

int gnnd_exact_knn(const void* vec, int64_t n, int32_t d, int32_t metric, const int32_t* queries,
                   int64_t nq, int32_t K, int32_t* ids_out, void* dist_out, void* stream) {
  if (!vec || !queries || !ids_out || !dist_out)
    return fail(nullptr, GNND_EINVAL, "NULL pointer argument");
  if (metric < GNND_L2SQ_F32 || metric > GNND_COSINE_F32)
    return fail(nullptr, GNND_EINVAL, "unknown metric");
  if (n < 2 || n > ((int64_t)1 << 30) || d < 1 || nq < 0 || K < 1 || K > 64)
    return fail(nullptr, GNND_EINVAL, "need 2 <= n <= 2^30, d >= 1, nq >= 0, 1 <= K <= 64");
  if ((uintptr_t)vec & 15) return fail(nullptr, GNND_EINVAL, "vectors must be 16-byte aligned");
  hipError_t e = launch_exact_knn(vec, n, d, metric, queries, nq, K, ids_out, dist_out,
                                  (hipStream_t)stream);
  return e == hipSuccess ? GNND_OK : hip_fail(nullptr, e, "exact_knn kernel");
}

}  // extern "C"
