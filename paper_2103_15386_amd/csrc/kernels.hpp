// Host-callable launchers of the GNND kernels (one per pipeline stage) and the
// device-pointer bundle they work on.  Every launcher enqueues on `st` and
// returns the hipGetLastError() of its launches.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gnnd {

enum : int {
  C_INSERTS = 0, C_EVALS = 1, C_SUMNEW = 2, C_SUMOLD = 3, C_PROPS = 4,
  C_OVERFLOW = 5,  // proposals that found their destination segment full (must stay 0)
  C_PASSED = 6,    // results that survived the early drop and went to the update
  C_SLOTS = 8
};
constexpr int kStripes = 64;  // counters are striped to spread same-address atomics

// One 64-bit word per destination serves the hand-out of results: the low
// kSlotCountBits bits count the results received so far, the rest is the first
// slot of the destination's segment.  A single returning atomic add yields both.
constexpr int kSlotCountBits = 24;
constexpr uint64_t kSlotCountMask = (1ull << kSlotCountBits) - 1;

// What the join gathers per sampled object besides its vector, kept small (8
// bytes, 8 MB per million nodes) so that the array stays cache resident: the
// distance code of its list's last entry (nothing farther can enter) and the
// squared norm of its int8 row (int8 join) or the bits of the float32 squared
// norm of its row (float32 matrix-core join).
struct alignas(8) NodeMeta {
  uint32_t kth;
  int32_t norm;
};

// Everything lives in the caller's workspace; sizes in elements.
struct DevState {
  uint64_t* G;         // n*k packed entries, row per node, ascending
  NodeMeta* meta;      // n: per-node record gathered by the join (see NodeMeta)
  int32_t* snew;       // n*2p NEW sample lists
  int32_t* sold;       // n*2p OLD sample lists
  int32_t* cnew;       // n list sizes
  int32_t* cold;       // n
  uint64_t* roff_new;  // n+1 offsets into csr_new
  uint64_t* roff_old;  // n+1
  int32_t* csr_new;    // n*p reverse candidates grouped by target
  int32_t* csr_old;    // n*p
  uint32_t* capn;      // n: upper bound of the proposals a node can receive as a NEW sample
  uint32_t* capo;      // n: ... as an OLD sample
  uint64_t* pslot;     // n: (segment start << 24) | proposals received; rewritten by every sampling
  uint64_t* poff;      // n+1 segment offsets into bins (exclusive scan of capn + capo)
  uint64_t* bins;      // n*6p packed proposals, one segment per destination
  uint64_t* scan_tmp;  // block sums of the scans
  uint64_t* counters;  // kStripes * C_SLOTS
  uint64_t* aside;     // merge only: n * floor(k/2) set-aside entries
  int8_t* shadow;      // matrix-core path: n rows of dpad int8 (value - 128), zero padded
  uint32_t* bk_cnt;    // 2 x 4096 bucket sizes of the bucketed reverse-candidate sort
  uint64_t* bk_off;    // 2 x 4097 bucket offsets
  // staged hand-out of the matrix-core join (NULL when results are handed on one by one):
  // results leave the join grouped by bucket of destinations, then a second pass moves
  // them into the destinations' segments of `bins`
  uint64_t* stg_ent;   // slots: staged results (see stage_record), bucket regions laid out like bins
  unsigned long long* stg_cur;  // kStageBuckets: results that have reached each bucket region
  // float32 matrix-core join and staged int8 join (NULL when neither is in use): the nodes
  // that have work to do, listed per class of node - kNodeClassesMax lists of n places, of
  // which the float join uses kGramClasses and the int8 join three - and the lists' lengths
  int32_t* cls_nodes;
  uint32_t* cls_count;
};
constexpr int kGramClasses = 7;
constexpr int kNodeClassesMax = 7;

// Staged hand-out: destinations are cut into at most kStageBuckets buckets of 2^tb
// consecutive ids; a workgroup of the join keeps kStageSlots results per bucket in LDS.
// A staged result is one 64-bit word: distance code (32) | destination inside its bucket
// (12) | object id (20), which is what limits the staged form to 2^20 nodes.
constexpr int kStageBuckets = 256;
constexpr int kStageSlots = 64;
constexpr int kStageIdBits = 20;
constexpr int64_t kStageMaxNodes = (int64_t)1 << kStageIdBits;
inline int stage_bucket_bits(int64_t n) {
  int tb = 0;
  while (((n + ((int64_t)1 << tb) - 1) >> tb) > kStageBuckets) ++tb;
  return tb;
}

struct Shape {
  int64_t n;
  int32_t d, k, p, metric;
  int64_t split;  // merge: first id of the second set; otherwise n
  const void* vec_a;
  const void* vec_b;
  int32_t all_pairs;  // 1: every evaluated pair is proposed (ablation), 0: nearest partners only
  const float* norms = nullptr;  // squared norm per node, where metric or join need it
  int32_t segments = 1;  // > 1: the list is k / 32 segments, object v lives in segment v % segments
  // slots of the proposal array: per appearance in a NEW list two results (all pairs: one per
  // possible partner, 2 * 2p - 1), in an OLD list one (all pairs: 2p); at most 2np appearances each
  __host__ __device__ int64_t slots_new_per_appearance() const {
    return all_pairs ? 4 * p - 1 : 2;
  }
  __host__ __device__ int64_t slots_old_per_appearance() const { return all_pairs ? 2 * p : 1; }
  __host__ __device__ int64_t slots() const {
    return n * 2 * p * (slots_new_per_appearance() + slots_old_per_appearance());
  }
};

// Grid of `blocks` workgroups, folded into two dimensions beyond 2^22 (device side:
// block_linear()); the fold may add up to 2^22 - 1 workgroups past the end.
inline dim3 grid_blocks(int64_t blocks) {
  constexpr int64_t kRow = (int64_t)1 << 22;
  if (blocks <= kRow) return dim3((unsigned)(blocks > 0 ? blocks : 1));
  return dim3((unsigned)kRow, (unsigned)((blocks + kRow - 1) / kRow));
}

hipError_t launch_init_random(const Shape& sh, const DevState& ds, uint64_t seed, hipStream_t st);
// squared norms of all rows, one fused multiply-add per dimension in dimension order
hipError_t launch_row_norms(const Shape& sh, float* norms, hipStream_t st);
hipError_t launch_sample(const Shape& sh, const DevState& ds, uint64_t seed, uint32_t iter,
                         hipStream_t st);
hipError_t launch_join(const Shape& sh, const DevState& ds, int path, bool merge_mode,
                       hipStream_t st);
// The float32 matrix-core join reads a sample's squared norm from its NodeMeta record (bits of
// the float in `norm`): copied there from sh.norms once the join path is chosen.
hipError_t launch_gram_norms(const Shape& sh, const DevState& ds, hipStream_t st);
// float32 vectors, metrics that are functions of an inner product and the norms (sh.norms
// must be set): inner products on the matrix cores, canonical distances for the results
hipError_t launch_join_gram(const Shape& sh, const DevState& ds, bool merge_mode, hipStream_t st);
// results are staged per bucket when ds.stg_ent is set, handed on one by one otherwise;
// `after_join` (may be NULL) is recorded behind the cross-matching kernel, in front of the
// pass that moves staged results into the destinations' segments.  `first_look`: the graph is
// a fresh random one (first iteration) - a hint that selects a form of the staged join that
// leaves the lists' thresholds to the second pass; same results with or without it
hipError_t launch_join_mfma(const Shape& sh, const DevState& ds, bool merge_mode, bool first_look,
                            hipStream_t st, hipEvent_t after_join = nullptr);
hipError_t launch_pack_i8(const Shape& sh, const DevState& ds, int* bad_flag_dev, hipStream_t st);
hipError_t launch_init_random_i8(const Shape& sh, const DevState& ds, uint64_t seed,
                                 hipStream_t st);
hipError_t launch_sample_buckets(const Shape& sh, const DevState& ds, hipStream_t st);
// sample lists of 65..128 objects (p > 32): reverse selection and the join for long lists
hipError_t launch_rev_select_long(const Shape& sh, const DevState& ds, uint64_t seed,
                                  uint32_t iter, hipStream_t st);
hipError_t launch_join_long(const Shape& sh, const DevState& ds, bool merge_mode, hipStream_t st);
hipError_t launch_update(const Shape& sh, const DevState& ds, hipStream_t st);
// lists of 65..128 entries (two per lane); the launchers above forward to these
hipError_t launch_init_random_wide(const Shape& sh, const DevState& ds, uint64_t seed,
                                   hipStream_t st);
hipError_t launch_update_wide(const Shape& sh, const DevState& ds, hipStream_t st);
// segmented lists (sh.segments > 1); the launchers above forward to these as well
hipError_t launch_init_random_segmented(const Shape& sh, const DevState& ds, uint64_t seed,
                                        hipStream_t st);
hipError_t launch_update_segmented(const Shape& sh, const DevState& ds, hipStream_t st);
hipError_t launch_get_graph(const Shape& sh, const DevState& ds, int32_t* ids, void* dist,
                            uint8_t* isnew, int32_t id_offset, hipStream_t st);
hipError_t launch_set_graph(const Shape& sh, const DevState& ds, const int32_t* ids,
                            const void* dist, const uint8_t* isnew, int* bad_flag_dev,
                            hipStream_t st);
hipError_t launch_get_proposals(const Shape& sh, const DevState& ds, int32_t* u, int32_t* v,
                                void* dist, hipStream_t st);
struct MergeIds;
hipError_t launch_merge_init(const Shape& sh, const DevState& ds, uint64_t seed,
                             const MergeIds& mi, const int32_t* ids1, const void* dist1,
                             const int32_t* ids2, const void* dist2, hipStream_t st);
hipError_t launch_merge_final(const Shape& sh, const DevState& ds, const MergeIds& mi,
                              int32_t* ids_out, void* dist_out, hipStream_t st);
// the same on the int8 rows of the matrix-core path (exact integers either way)
hipError_t launch_merge_init_i8(const Shape& sh, const DevState& ds, uint64_t seed,
                                const MergeIds& mi, const int32_t* ids1, const void* dist1,
                                const int32_t* ids2, const void* dist2, hipStream_t st);
hipError_t launch_merge_init_wide(const Shape& sh, const DevState& ds, uint64_t seed,
                                  const MergeIds& mi, const int32_t* ids1, const void* dist1,
                                  const int32_t* ids2, const void* dist2, hipStream_t st);
hipError_t launch_merge_final_wide(const Shape& sh, const DevState& ds, const MergeIds& mi,
                                   int32_t* ids_out, void* dist_out, hipStream_t st);
hipError_t launch_exact_knn(const void* vec, int64_t n, int32_t d, int32_t metric,
                            const int32_t* queries, int64_t nq, int32_t K, int32_t* ids_out,
                            void* dist_out, hipStream_t st);
hipError_t launch_zero_u32(uint32_t* p, size_t count, hipStream_t st);
hipError_t launch_copy_u64(uint64_t* dst, const uint64_t* src, size_t count, hipStream_t st);

// Exclusive scan of `count` uint32 into uint64 offsets out[0..count] (out[count] = total).
// (in2 may be NULL; otherwise the scanned values are in[i] + in2[i])
hipError_t launch_scan(const uint32_t* in, const uint32_t* in2, uint64_t* out, uint64_t* packed,
                       uint64_t* counters, uint64_t* tmp,
                       int64_t count, hipStream_t st);
size_t scan_tmp_elems(int64_t count);

}  // namespace gnnd
