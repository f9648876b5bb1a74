// Cross-matching (Sec. 4.2) and nearest-object search (Sec. 4.3, Alg. 2) on
// the matrix cores, for byte-valued data: one 64-lane wavefront per node.
//
// The node's <= 64 NEW and <= 64 OLD sample vectors are read straight from HBM
// into MFMA operand registers (16 bytes per lane per 32-dimension step; a 128 B
// row is one cache line).  Vectors are stored shifted to int8 (x - 128), which
// leaves differences unchanged, so with the Gram block G = A.B^T from
// v_mfma_i32_32x32x32_i8 the squared distance is |a|^2 + |b|^2 - 2 G, exact in
// int32.  A 32x32 accumulator tile keeps one column per lane, so "nearest row
// object for every column object" is a per-lane min over 16 registers plus one
// half-wave swap; the tile is computed in both orientations where both
// directions are needed (NEW->OLD and OLD->NEW) instead of reducing across
// lanes.  Sample lists are sorted by id, so the row position inside a list
// breaks distance ties exactly like the id does.
#include <type_traits>

#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kMB = 256;  // 4 waves = 4 nodes in flight per workgroup
constexpr int64_t kJoinGrid = 256 * 3 * 2;  // 256 CUs x 3 resident workgroups x 2
// staged hand-out: one workgroup of 8 waves per CU (2 per SIMD: the staging code needs the registers) shares the staging area
constexpr int kStagedWaves = 8;       // four operand blocks: 2 wavefronts per SIMD
constexpr int kStagedWavesSlim = 12;  // three operand blocks: 3 wavefronts per SIMD
constexpr int kMBStaged = kStagedWaves * kWave;
constexpr int32_t kFar = 1 << 24;  // "norm" of an absent row: above every real distance

// Convert float32 rows holding integers 0..255 (or uint8 rows) to int8 rows
// (value - 128) of `dpad` bytes, zero padded, and store the squared norm of
// the shifted row.  `bad` is raised when a float is not such an integer.
template <typename T>
__global__ __launch_bounds__(256) void k_pack_i8(const void* vec_a, const void* vec_b,
                                                 int64_t split, int64_t n, int d, int dpad,
                                                 int8_t* shadow, NodeMeta* meta, int* bad) {
  const int lane = lane_id();
  const int64_t row = block_linear() * 4 + wave_id();
  if (row >= n) return;
  const T* src = row < split ? reinterpret_cast<const T*>(vec_a) + row * d
                             : reinterpret_cast<const T*>(vec_b) + (row - split) * d;
  int32_t acc = 0;
  bool is_bad = false;
  for (int j = lane; j < dpad; j += kWave) {
    int32_t q = 0;
    if (j < d) {
      float f = (float)src[j];
      int32_t iv = (int32_t)f;
      if (!(f >= 0.f && f <= 255.f) || (float)iv != f) is_bad = true;
      q = iv - 128;
      acc += q * q;
    }
    shadow[row * dpad + j] = (int8_t)q;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
  if (lane == 0) meta[row].norm = acc;
  if (__ballot(is_bad) != 0ull && lane == 0) atomicOr(bad, 1);
}

// The same for uint8 rows whose length is a multiple of 16: a lane moves 16
// bytes (x - 128 is x ^ 0x80 in every byte), C = dpad / 16 neighbouring lanes
// share a row, so loads and stores of a wavefront are contiguous.
__global__ __launch_bounds__(256) void k_pack_u8_wide(const uint8_t* vec_a, const uint8_t* vec_b,
                                                      int64_t split, int64_t n, int d, int dpad,
                                                      int8_t* shadow, NodeMeta* meta) {
  const int lane = lane_id();
  const int C = dpad >> 4, per_wave = kWave / C;
  const int grp = lane / C, sub = lane - grp * C;
  const int64_t row = (block_linear() * 4 + wave_id()) * per_wave + grp;
  const bool on = grp < per_wave && row < n;
  int32_t part = 0;
  if (on) {
    v4i q = {0, 0, 0, 0};
    if (16 * sub < d) {
      const uint8_t* src = row < split ? vec_a + row * d : vec_b + (row - split) * d;
      q = *reinterpret_cast<const v4i*>(src + 16 * sub);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        q[t] ^= (int)0x80808080;
        part = __builtin_amdgcn_sdot4(q[t], q[t], part, false);
      }
    }
    *reinterpret_cast<v4i*>(shadow + row * dpad + 16 * sub) = q;
  }
  int32_t total = 0;
  for (int t = 0; t < C; ++t) total += __shfl(part, (grp * C + t) & 63, kWave);
  if (on && sub == 0) meta[row].norm = total;
}

// Exact squared distances |a|^2 + |b|^2 - 2 a.b (four products per v_dot4) on
// the int8 rows, from node s to one object per lane: `id` of lanes < count.
// A row is C = dpad / 16 <= 8 chunks of 16 bytes; the C lanes of a group read
// one object's row as one contiguous line (64 / C objects per load), multiply
// it with the node's own chunk and add up across the group; the sums are then
// handed to the lanes that hold the objects.  All 64 lanes call it together;
// lanes >= count get 0.
__device__ inline int32_t wave_distances_i8(const int8_t* __restrict__ shadow,
                                            const NodeMeta* meta, int dpad, int64_t s, uint32_t id,
                                            int count, int lane) {
  const int C = dpad >> 4, per_load = kWave / C;
  const int grp = lane / C, sub = lane - grp * C;
  const bool lane_used = grp < per_load;  // C = 6 leaves four lanes without a group
  const bool pow2 = (C & (C - 1)) == 0;
  const v4i x = *reinterpret_cast<const v4i*>(shadow + s * dpad + 16 * sub);
  const int32_t norm_s = meta[s].norm;
  // (the objects' norms come from their rows, which are here anyway: a gather of the stored
  // norm would be a second scattered access per object)
  int32_t dot = 0, norm_id = 0;
  for (int r0 = 0; r0 < count; r0 += per_load) {
    const int j = r0 + grp;  // the object this group reads
    const bool act = lane_used && j < count;
    const uint32_t nid = __shfl(id, act ? j : 0, kWave);
    int32_t part = 0, part_sq = 0;
    if (act) {
      const v4i y = *reinterpret_cast<const v4i*>(shadow + (int64_t)nid * dpad + 16 * sub);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        part = __builtin_amdgcn_sdot4(x[t], y[t], part, false);
        part_sq = __builtin_amdgcn_sdot4(y[t], y[t], part_sq, false);
      }
    }
    int32_t total = part, total_sq = part_sq;
    if (pow2) {  // groups are aligned blocks of 2, 4 or 8 lanes: butterfly sum
      if (C > 1) {
        total += (int32_t)xor_lanes((uint32_t)total, 1, lane);
        total_sq += (int32_t)xor_lanes((uint32_t)total_sq, 1, lane);
      }
      if (C > 2) {
        total += (int32_t)xor_lanes((uint32_t)total, 2, lane);
        total_sq += (int32_t)xor_lanes((uint32_t)total_sq, 2, lane);
      }
      if (C > 4) {
        total += (int32_t)xor_lanes((uint32_t)total, 4, lane);
        total_sq += (int32_t)xor_lanes((uint32_t)total_sq, 4, lane);
      }
    } else {
      for (int off = 1; off < C; ++off) {
        int o = sub + off;
        o = o >= C ? o - C : o;
        total += __shfl(part, (grp * C + o) & 63, kWave);
        total_sq += __shfl(part_sq, (grp * C + o) & 63, kWave);
      }
    }
    // object j = lane sits in group lane - r0
    const int32_t got = __shfl(total, ((lane - r0) * C) & 63, kWave);
    const int32_t got_sq = __shfl(total_sq, ((lane - r0) * C) & 63, kWave);
    if (lane >= r0 && lane < r0 + per_load) {
      dot = got;
      norm_id = got_sq;
    }
  }
  return lane < count ? norm_s + norm_id - 2 * dot : 0;
}

// Alg. 1, first loop, on the int8 rows: k distinct random neighbours per node,
// exact distances, sorted ascending by (distance, id), flagged NEW.  One
// wavefront per node.
template <bool FCODE>
__global__ __launch_bounds__(256) void k_init_random_i8(const int8_t* __restrict__ shadow,
                                                        NodeMeta* meta, int dpad, int64_t n, int k,
                                                        uint64_t base_hash, uint64_t* G) {
  const int lane = lane_id();
  const int64_t s = block_linear() * 4 + wave_id();
  if (s >= n) return;
  // the list for one id per lane, ascending
  auto list_of = [&](uint32_t id) {
    const int32_t dist = wave_distances_i8(shadow, meta, dpad, s, id, k, lane);
    uint64_t e = kKeyMax;
    if (lane < k) e = make_entry(FCODE ? ord_f32((float)dist) : ord_i32(dist), id, 1u);
    return wave_sort_upto(e, lane, k);
  };
  // First attempts of all slots at once.  Whether they are valid (pairwise distinct,
  // none the node itself) shows after the sort: equal ids have equal distances and
  // end up next to each other.  Only then the slot-by-slot rule has to run.
  uint64_t e = list_of(draw_first(base_hash, (uint32_t)s, (uint32_t)n, 0u, lane));
  const uint64_t prev = __shfl_up(e, 1, kWave);
  const bool bad = lane < k && (entry_id(e) == (uint32_t)s ||
                                (lane > 0 && entry_id(e) == entry_id(prev)));
  if (__ballot(bad) != 0ull)
    e = list_of(draw_slot_by_slot(base_hash, (uint32_t)s, k, (uint32_t)n, 0u, (uint32_t)s, lane));
  if (lane < k) G[s * k + lane] = e;
  if (lane == k - 1) meta[s].kth = entry_code(e);
}

// GGM, Alg. 3 "Divide" + "Append" on the int8 rows: keep the first ceil(k/2)
// entries (OLD), set the rest aside, refill with floor(k/2) random objects of
// the other set (NEW, exact distances) and restore the (distance, id) order.
template <bool FCODE>
__global__ __launch_bounds__(256) void k_merge_init_i8(const int8_t* __restrict__ shadow,
                                                       NodeMeta* meta, int dpad, int64_t n,
                                                       MergeIds mi, int k, uint64_t base_hash,
                                                       const int32_t* ids1, const void* dist1,
                                                       const int32_t* ids2, const void* dist2,
                                                       uint64_t* G, uint64_t* aside) {
  const int lane = lane_id();
  const int64_t s = block_linear() * 4 + wave_id();
  if (s >= n) return;
  const int64_t n1 = mi.n1;
  const bool first = s < n1;
  const int64_t loc = first ? s : s - n1;
  const int32_t* sid = (first ? ids1 : ids2) + loc * k;
  const void* sdist = first ? dist1 : dist2;
  const int keep = (k + 1) / 2, fill = k / 2;
  uint32_t id_in = 0, code_in = 0;
  if (lane < k) {
    id_in = mi.to_internal(sid[lane]);  // collection id -> numbering of this merge
    code_in = FCODE ? ord_f32(reinterpret_cast<const float*>(sdist)[loc * k + lane])
                    : ord_i32(reinterpret_cast<const int32_t*>(sdist)[loc * k + lane]);
  }
  if (lane >= keep && lane < k) aside[s * fill + (lane - keep)] = make_entry(code_in, id_in, 0u);
  const uint32_t draw = draw_distinct(base_hash, (uint32_t)s, fill,
                                      (uint32_t)(first ? n - n1 : n1), first ? (uint32_t)n1 : 0u,
                                      0xffffffffu, lane);
  const int32_t dist = wave_distances_i8(shadow, meta, dpad, s, draw, fill, lane);
  const uint32_t code_of_draw = FCODE ? ord_f32((float)dist) : ord_i32(dist);
  const int src = lane - keep;
  const uint32_t did = __shfl(draw, src < 0 ? 0 : src, kWave);
  const uint32_t code = __shfl(code_of_draw, src < 0 ? 0 : src, kWave);
  uint64_t e = kKeyMax;
  if (lane < keep) e = make_entry(code_in, id_in, 0u);
  else if (lane < k) e = make_entry(code, did, 1u);
  e = wave_sort(e, lane);
  if (lane < k) G[s * k + lane] = e;
  if (lane == k - 1) meta[s].kth = entry_code(e);
}

// Best row per column of one 32x32 accumulator tile.  For row r the LDS array
// holds negR = -((norm_r << 6) | position_r); then t = (G << 7) + negR is
// -(((norm_r - 2 G) << 6) | position_r), so the maximum of t over the rows is
// the row with the smallest (norm_r - 2 G), ties to the smallest position -
// one shift-add and half a max3 per accumulator register.  Adding the column's
// own norm to ((-t) >> 6) gives the squared distance; |.| stays below 2^31
// because norms are below 2^22 (absent rows: 2^24 with G = 0).  Rows flagged
// in `excl` are skipped.  Row of register r for this lane: 8*(r/4) + 4*half + r%4.
constexpr int32_t kNone = (int32_t)0x80000000;

template <bool MASKED>
__device__ inline int32_t tile_col_best(const v16i& g, const int32_t* negr_lds, int half,
                                        uint32_t excl) {
  int32_t best = kNone;
  const uint32_t ex = excl >> (4 * half);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int4 nr = *reinterpret_cast<const int4*>(negr_lds + 8 * q + 4 * half);
    const int32_t negr[4] = {nr.x, nr.y, nr.z, nr.w};
    int32_t t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      t[i] = (int32_t)(((uint32_t)g[4 * q + i] << 7) + (uint32_t)negr[i]);
      if (MASKED) t[i] = (ex & (1u << (8 * q + i))) ? kNone : t[i];
    }
    best = max(best, max(t[0], t[1]));
    best = max(best, max(t[2], t[3]));
  }
  return best;
}

__device__ inline int32_t both_halves_max(int32_t x) {
  auto sw = __builtin_amdgcn_permlane32_swap((uint32_t)x, (uint32_t)x, false, false);
  int32_t a = (int32_t)sw[0], b = (int32_t)sw[1];
  return a > b ? a : b;
}

typedef uint64_t EntryPair __attribute__((ext_vector_type(2), aligned(8)));

struct Operand {
  v4i k[4];  // 4 steps of 32 dimensions, 16 bytes of this lane each
};

template <int KSTEPS>
__device__ inline Operand load_block(const int8_t* shadow, int dpad, int32_t id, int half) {
  Operand o;
#pragma unroll
  for (int s = 0; s < 4; ++s) o.k[s] = v4i{0, 0, 0, 0};
  if (id >= 0) {
    const int8_t* row = shadow + (int64_t)id * dpad + 16 * half;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) o.k[s] = *reinterpret_cast<const v4i*>(row + 32 * s);
  }
  return o;
}

template <int KSTEPS>
__device__ inline v16i gram(const Operand& rows, const Operand& cols) {
  v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s)
    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(rows.k[s], cols.k[s], acc, 0, 0, 0);
  return acc;
}

// FCODE: distances are reported as float32 codes (float input data) instead of
// int32 codes.  MERGE: GGM mode - no NEW x NEW, only pairs from different sets.
//
// Each wavefront walks over nodes s, s + W, s + 2W, ... (W = wavefronts in the
// grid) as a software pipeline, because a node costs three dependent memory
// round trips (sample ids -> vector rows -> result slots): while the tiles of
// node i are evaluated the ids of node i+1 are already in flight, and as soon
// as the last tile has consumed the operand registers the rows of node i+1 are
// requested, before the results of node i are handed out.
// STAGED: results are not handed to their destinations one by one (one returning
// device-wide atomic and one scattered 8-byte store each - the rate of those atomics
// was what the kernel ran at) but collected per workgroup in LDS, kStageSlots places
// for each of <= kStageBuckets buckets of consecutive destination ids, and written
// out bucket by bucket: one atomic and one contiguous piece per bucket and flush.
// The bucket regions tile an array shaped like `bins` (a bucket's region starts where
// the segment of its first destination starts, so it can hold whatever its
// destinations can receive); k_result_csr then moves every result into its
// destination's segment.  A result that finds its bucket's places taken goes to the
// bucket's region directly.
//
// The waves of a workgroup run at their own pace, so a flush is a rendezvous: every
// wave looks at the fill count after each node and joins the flush once it has reached
// the threshold (the count only falls inside a flush, so every wave gets there); a wave
// that has run out of nodes keeps joining flushes until all waves have run out.
struct StageArgs {
  uint64_t* ent;            // bucket regions: staged results
  unsigned long long* cur;  // per bucket: results written to its region so far
  const uint64_t* poff;     // segment offsets of the destinations (n + 1)
  int tb, nb;               // log2(destinations per bucket), number of buckets
  uint32_t threshold;       // fill count that triggers a flush
  const int32_t* nodes;     // kJoinShapes lists of n places: the nodes of each shape
  const uint32_t* count;    // their lengths
  bool count_passed;        // false when the pass behind the join counts what passes
};
constexpr size_t kStageLdsBytes = (size_t)kStageBuckets * kStageSlots * 8 + kStageBuckets * 20 + 16;
// a staged result: distance code | destination inside its bucket | object id
__device__ inline uint64_t stage_record(uint64_t entry, uint32_t dest, int tb) {
  return (entry & 0xffffffff00000000ull) | ((uint64_t)(dest & ((1u << tb) - 1u)) << kStageIdBits) |
         (uint64_t)entry_id(entry);
}

// Squared norm of the row this lane's sample stands for, from the operand registers: sample
// `lane` of a list is row lane % 32 of block lane / 32, and lanes l and l + 32 hold the two
// halves of row l of both blocks.
template <int KSTEPS>
__device__ inline int32_t half_row_sq(const Operand& o) {
  int32_t acc = 0;
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_sdot4(o.k[s][i], o.k[s][i], acc, false);
  return acc;
}
template <int KSTEPS>
__device__ inline int32_t sample_norm(const Operand& b0, const Operand& b1, int half, int lane) {
  const int32_t p0 = half_row_sq<KSTEPS>(b0), p1 = half_row_sq<KSTEPS>(b1);
  const int32_t mine = half ? p1 : p0, give = half ? p0 : p1;
  return mine + (int32_t)xor_lanes((uint32_t)give, 32, lane);
}

// LEAN: the form for a launch in which the thresholds of the lists
// decide little and the nodes have few OLD samples - the first iteration on a random graph,
// where every result passes and a node's time is the time the memory system needs for its
// scattered lines.  The 8-byte (threshold, norm) records, one more scattered line per sampled
// object, are not read: the norms come from the operand registers and every result found is
// handed on; k_result_csr<true> then applies the thresholds (staged hand-out; with the direct
// hand-out the list update drops what cannot enter), so the same results reach the lists.
// Right for any input; faster only where the saved reads outweigh the extra arithmetic and
// the larger flow of results.
// SHAPE (staged hand-out only): which of the four operand blocks of 32 rows a node fills.
// 0: any (NEW 0..31, NEW 32..63, OLD 0..31, OLD 32..63); 1: at most 32 OLD samples; 2: at
// most 32 NEW samples.  Most nodes are of shape 1 (early iterations: many NEW, few OLD) or 2
// (late ones); without the fourth block's 16 registers the kernel fits 3 wavefronts per SIMD,
// which hide the per-node chain wait -> evaluate -> hand on better than 2 do (6 to 12 % less
// time per iteration).  k_join_shapes lists the nodes of each shape (those with nothing to
// evaluate are in no list) and every build runs over its own list.
constexpr int kJoinShapes = 3;
__host__ __device__ constexpr int join_list_of_shape(int shape) { return shape == 0 ? 2 : shape - 1; }
__host__ __device__ constexpr int join_waves(bool staged, int shape) {
  return staged ? (shape ? kStagedWavesSlim : kStagedWaves) : kMB / kWave;
}

template <int KSTEPS, bool FCODE, bool MERGE, bool STAGED, bool LEAN = false, int SHAPE = 0>
__global__ __launch_bounds__(join_waves(STAGED, SHAPE) * kWave)
__attribute__((amdgpu_waves_per_eu(STAGED && !SHAPE ? 2 : 3, STAGED && !SHAPE ? 2 : 3))) void k_join_mfma(
    const int8_t* __restrict__ shadow, const NodeMeta* __restrict__ meta, int dpad, int64_t n,
    int p, int64_t split, const int32_t* __restrict__ snew, const int32_t* __restrict__ sold,
    uint64_t* pslot, uint64_t slots, uint64_t* __restrict__ bins, uint64_t* counters,
    StageArgs sa) {
  constexpr int WAVES = join_waves(STAGED, SHAPE);
  constexpr bool kHasN1 = SHAPE != 2, kHasO1 = SHAPE != 1;
  static_assert(STAGED || SHAPE == 0, "shapes come with the node lists of the staged form");
  // per wave, for the 128 rows (NEW 0..63, OLD 64..127): -((norm << 6) | position), the ids
  // (absent = INT_MAX so that both halves stay ascending), and a scratch row
  __shared__ __attribute__((aligned(16))) int32_t s_norm[WAVES][128];
  __shared__ int32_t s_id[WAVES][128];
  __shared__ int32_t s_eq[WAVES][64];
  extern __shared__ __attribute__((aligned(16))) unsigned char stage_raw[];
  uint64_t* const st_ent = reinterpret_cast<uint64_t*>(stage_raw);
  uint64_t* const st_region = st_ent + kStageBuckets * kStageSlots;
  uint64_t* const st_gbase = st_region + kStageBuckets;
  uint32_t* const st_cnt = reinterpret_cast<uint32_t*>(st_gbase + kStageBuckets);
  uint32_t* const st_fill = st_cnt + kStageBuckets;  // [0] results staged, [1] waves out of nodes
  // (the wave index as a vector value: measured 3 % faster here than the scalar form)
  const int wave = threadIdx.x >> 6, lane = lane_id(), half = lane >> 5, col = lane & 31;
  // (with lists n <= 2^20: places, node numbers and offsets into the sample lists fit 32 bits)
  using node_t = typename std::conditional<STAGED, int32_t, int64_t>::type;
  const node_t W = (node_t)gridDim.x * WAVES;
  // place `pos` of this build's list of nodes (staged) / of all nodes (direct)
  node_t pos = (node_t)blockIdx.x * WAVES + wave;
  const node_t places = STAGED ? (node_t)sa.count[join_list_of_shape(SHAPE)] : (node_t)n;
  const int32_t* const list = STAGED ? sa.nodes + (int64_t)join_list_of_shape(SHAPE) * n : nullptr;
  auto node_at = [&](node_t at) -> node_t {  // -1 beyond the end
    if (at >= places) return (node_t)-1;
    return STAGED ? (node_t)list[at] : (node_t)at;
  };
  if (!STAGED && pos >= n) return;
  if (STAGED) {
    for (int b = threadIdx.x; b < sa.nb; b += WAVES * kWave) {
      st_cnt[b] = 0;
      const int64_t first = (int64_t)b << sa.tb;
      st_region[b] = sa.poff[first < n ? first : n];
    }
    if (threadIdx.x == 0) st_fill[0] = st_fill[1] = 0;
    __syncthreads();
  }
  // One flush (all waves of the workgroup together).  Returns true when every wave has
  // run out of nodes, i.e. when this was the last one.
  auto flush = [&]() -> bool {
    __syncthreads();  // nobody is adding results any more
    const uint32_t out_of_nodes = *reinterpret_cast<volatile uint32_t*>(st_fill + 1);
    for (int b = threadIdx.x; b < sa.nb; b += WAVES * kWave) {
      const uint32_t c = st_cnt[b] < (uint32_t)kStageSlots ? st_cnt[b] : (uint32_t)kStageSlots;
      st_gbase[b] = c ? atomicAdd(&sa.cur[b], (unsigned long long)c) : 0ull;
    }
    __syncthreads();
    // a wave per bucket: its results leave as one contiguous piece
    for (int b = wave; b < sa.nb; b += WAVES) {
      const uint32_t c = st_cnt[b] < (uint32_t)kStageSlots ? st_cnt[b] : (uint32_t)kStageSlots;
      const uint64_t at = st_region[b] + st_gbase[b] + (uint32_t)lane;
      if ((uint32_t)lane < c && at < slots) sa.ent[at] = st_ent[b * kStageSlots + lane];
    }
    __syncthreads();
    for (int b = threadIdx.x; b < sa.nb; b += WAVES * kWave) st_cnt[b] = 0;
    if (threadIdx.x == 0) st_fill[0] = 0;
    __syncthreads();
    return out_of_nodes == (uint32_t)WAVES;
  };
  // this node, the next one and the one after: sample ids are requested two nodes ahead
  node_t s = node_at(pos), s1 = node_at(pos + W), s2 = node_at(pos + 2 * W);
  const bool have_nodes = s >= 0;
  const int L = 2 * p;
  const bool in_list = lane < L;

  // unused list slots hold -1, so the ids alone say how long a list is
  int32_t id_new = (have_nodes && in_list) ? snew[s * L + lane] : -1;
  int32_t id_old = (have_nodes && in_list) ? sold[s * L + lane] : -1;
  int32_t nx_new = -1, nx_old = -1;
  if (s1 >= 0 && in_list) {
    nx_new = snew[s1 * L + lane];
    nx_old = sold[s1 * L + lane];
  }
  Operand N0, N1, O0, O1;
  uint2 m_new, m_old;
  auto request_rows = [&](int32_t idn, int32_t ido) {
    // block b of a list = its rows 32b..32b+31; lane (col, half) holds bytes
    // [32 step + 16 half, +16) of row `col` of the block for every step
    N0 = load_block<KSTEPS>(shadow, dpad, __shfl(idn, col, kWave), half);
    if (kHasN1) N1 = load_block<KSTEPS>(shadow, dpad, __shfl(idn, 32 + col, kWave), half);
    O0 = load_block<KSTEPS>(shadow, dpad, __shfl(ido, col, kWave), half);
    if (kHasO1) O1 = load_block<KSTEPS>(shadow, dpad, __shfl(ido, 32 + col, kWave), half);
    m_new = m_old = make_uint2(0u, (uint32_t)kFar);  // an absent sample: far from everything
    if (!LEAN) {  // one 8-byte gather per sampled object: list threshold and norm
      if (idn >= 0) m_new = *reinterpret_cast<const uint2*>(meta + idn);
      if (ido >= 0) m_old = *reinterpret_cast<const uint2*>(meta + ido);
    }
  };
  request_rows(id_new, id_old);

  while (have_nodes) {
    const int nn = __popcll(__ballot(id_new >= 0)), no = __popcll(__ballot(id_old >= 0));
    const bool do_nn = !MERGE && nn > 1;
    const bool active = nn > 0 && (do_nn || no > 0);
    uint2 cm_new = m_new, cm_old = m_old;  // this node's thresholds and norms
    if (LEAN && active) {  // (all lanes take part in the exchange between the halves)
      // (a block the shape does not have stands for samples that are absent)
      const uint32_t norm_new = (uint32_t)sample_norm<KSTEPS>(N0, kHasN1 ? N1 : N0, half, lane);
      if (id_new >= 0) cm_new.y = norm_new;
      if (no > 0) {  // uniform
        const uint32_t norm_old = (uint32_t)sample_norm<KSTEPS>(O0, kHasO1 ? O1 : O0, half, lane);
        if (id_old >= 0) cm_old.y = norm_old;
      }
    }
    int32_t a0 = kNone, a1 = kNone;  // NEW column blocks: nearest other NEW
    int32_t b0 = kNone, b1 = kNone;  // NEW column blocks: nearest OLD
    int32_t c0 = kNone, c1 = kNone;  // OLD column blocks: nearest NEW
    uint32_t dups = 0;
    uint32_t cls_new0 = 0, cls_new1 = 0, cls_old0 = 0, cls_old1 = 0;
    if (active) {
      s_norm[wave][lane] = -(int32_t)((cm_new.y << 6) | (uint32_t)lane);
      s_norm[wave][64 + lane] = -(int32_t)((cm_old.y << 6) | (uint32_t)lane);
      s_id[wave][lane] = id_new >= 0 ? id_new : 0x7fffffff;
      s_id[wave][64 + lane] = id_old >= 0 ? id_old : 0x7fffffff;
      s_eq[wave][lane] = -1;
      // the wave reads these back below: order its own LDS writes before its reads
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      // objects sampled both as NEW and as OLD: that pair is not a pair.  eq_old =
      // position in the OLD list of this lane's NEW object (or -1), and vice versa.
      // Both lists ascend, so each NEW lane binary-searches its id in the OLD list.
      int eq_old = -1, eq_new = -1;
      if (no > 0) {
        int lo = 0, hi = 64;  // lower bound of id_new in the OLD list, in [0, 64]
#pragma unroll
        for (int step = 0; step < 7; ++step) {
          const bool go = lo < hi;
          const int mid = (lo + hi) >> 1;  // <= 63 while lo < hi
          const bool below = go && s_id[wave][64 + (mid & 63)] < id_new;
          lo = below ? mid + 1 : lo;
          hi = (go && !below) ? mid : hi;
        }
        if (id_new >= 0 && lo < 64 && s_id[wave][64 + lo] == id_new) eq_old = lo;
        dups = (uint32_t)__popcll(__ballot(eq_old >= 0));
        if (dups) {
          if (eq_old >= 0) s_eq[wave][eq_old] = lane;
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          eq_new = s_eq[wave][lane];
        }
      }
      // per-lane exclusion masks (bit r = row r of the block is not a partner of
      // this lane's column object); lanes l and l+32 serve column l%32 of block 0,
      // results of block 1 are selected into lanes 32..63 at the end
      const int eq_old_c0 = __shfl(eq_old, col, kWave), eq_old_c1 = __shfl(eq_old, 32 + col, kWave);
      const int eq_new_c0 = __shfl(eq_new, col, kWave), eq_new_c1 = __shfl(eq_new, 32 + col, kWave);
      const int32_t rid_n0 = __shfl(id_new, col, kWave), rid_n1 = __shfl(id_new, 32 + col, kWave);
      const int32_t rid_o0 = __shfl(id_old, col, kWave), rid_o1 = __shfl(id_old, 32 + col, kWave);
      // merge mode: rows whose set equals the column object's set are excluded
      if (MERGE) {
        const uint64_t cn = __ballot(id_new >= 0 && (int64_t)id_new >= split);
        const uint64_t co = __ballot(id_old >= 0 && (int64_t)id_old >= split);
        cls_new0 = (uint32_t)cn; cls_new1 = (uint32_t)(cn >> 32);
        cls_old0 = (uint32_t)co; cls_old1 = (uint32_t)(co >> 32);
      }
      auto excl_rows = [&](int eq_row, int row_block, uint32_t cls_rows, int32_t col_id) {
        uint32_t m = 0;
        if (eq_row >= 0 && (eq_row >> 5) == row_block) m |= 1u << (eq_row & 31);
        if (MERGE) m |= ((int64_t)col_id >= split) ? cls_rows : ~cls_rows;
        return m;
      };
      const bool masked_no = MERGE || dups != 0;
      const int32_t* normN = s_norm[wave];
      const int32_t* normO = s_norm[wave] + 64;

      if (do_nn) {
        {  // rows N0, columns N0: the diagonal pairs an object with itself
          v16i g = gram<KSTEPS>(N0, N0);
          a0 = max(a0, tile_col_best<true>(g, normN, half, 1u << col));
        }
        if (kHasN1 && nn > 32) {
          {
            v16i g = gram<KSTEPS>(N1, N0);
            a0 = max(a0, tile_col_best<false>(g, normN + 32, half, 0u));
          }
          {
            v16i g = gram<KSTEPS>(N0, N1);
            a1 = max(a1, tile_col_best<false>(g, normN, half, 0u));
          }
          {
            v16i g = gram<KSTEPS>(N1, N1);
            a1 = max(a1, tile_col_best<true>(g, normN + 32, half, 1u << col));
          }
        }
      }
      if (no > 0) {
        // columns = NEW objects, rows = OLD objects: nearest OLD of every NEW
        {
          v16i g = gram<KSTEPS>(O0, N0);
          b0 = max(b0, masked_no ? tile_col_best<true>(g, normO, half,
                                                      excl_rows(eq_old_c0, 0, cls_old0, rid_n0))
                                 : tile_col_best<false>(g, normO, half, 0u));
        }
        if (kHasO1 && no > 32) {
          v16i g = gram<KSTEPS>(O1, N0);
          b0 = max(b0, masked_no ? tile_col_best<true>(g, normO + 32, half,
                                                      excl_rows(eq_old_c0, 1, cls_old1, rid_n0))
                                 : tile_col_best<false>(g, normO + 32, half, 0u));
        }
        if (kHasN1 && nn > 32) {
          {
            v16i g = gram<KSTEPS>(O0, N1);
            b1 = max(b1, masked_no ? tile_col_best<true>(g, normO, half,
                                                        excl_rows(eq_old_c1, 0, cls_old0, rid_n1))
                                   : tile_col_best<false>(g, normO, half, 0u));
          }
          if (kHasO1 && no > 32) {
            v16i g = gram<KSTEPS>(O1, N1);
            b1 = max(b1, masked_no ? tile_col_best<true>(g, normO + 32, half,
                                                        excl_rows(eq_old_c1, 1, cls_old1, rid_n1))
                                   : tile_col_best<false>(g, normO + 32, half, 0u));
          }
        }
        // columns = OLD objects, rows = NEW objects: nearest NEW of every OLD
        {
          v16i g = gram<KSTEPS>(N0, O0);
          c0 = max(c0, masked_no ? tile_col_best<true>(g, normN, half,
                                                      excl_rows(eq_new_c0, 0, cls_new0, rid_o0))
                                 : tile_col_best<false>(g, normN, half, 0u));
        }
        if (kHasN1 && nn > 32) {
          v16i g = gram<KSTEPS>(N1, O0);
          c0 = max(c0, masked_no ? tile_col_best<true>(g, normN + 32, half,
                                                      excl_rows(eq_new_c0, 1, cls_new1, rid_o0))
                                 : tile_col_best<false>(g, normN + 32, half, 0u));
        }
        if (kHasO1 && no > 32) {
          {
            v16i g = gram<KSTEPS>(N0, O1);
            c1 = max(c1, masked_no ? tile_col_best<true>(g, normN, half,
                                                        excl_rows(eq_new_c1, 0, cls_new0, rid_o1))
                                   : tile_col_best<false>(g, normN, half, 0u));
          }
          if (kHasN1 && nn > 32) {
            v16i g = gram<KSTEPS>(N1, O1);
            c1 = max(c1, masked_no ? tile_col_best<true>(g, normN + 32, half,
                                                        excl_rows(eq_new_c1, 1, cls_new1, rid_o1))
                                   : tile_col_best<false>(g, normN + 32, half, 0u));
          }
        }
      }
    }

    // ---- hand the results out: lane l answers for sample l of its list -------
    uint32_t found_total = 0, over_total = 0;
    bool pass[3];
    uint64_t entry[3];
    int32_t self[3];
    if (active) {
      // combine the two row halves; lanes 0..31 take column block 0, lanes 32..63 block 1
      a0 = both_halves_max(a0); a1 = both_halves_max(a1);
      b0 = both_halves_max(b0); b1 = both_halves_max(b1);
      c0 = both_halves_max(c0); c1 = both_halves_max(c1);
      const int32_t res3[3] = {half ? a1 : a0, half ? b1 : b0, half ? c1 : c0};
#pragma unroll
      for (int kind = 0; kind < 3; ++kind) {
        const int32_t res = -res3[kind];  // ((row_norm - 2 G) << 6) | row position
        self[kind] = kind == 2 ? id_old : id_new;
        const uint2 cm = kind == 2 ? cm_old : cm_new;
        const int32_t part = res >> 6;  // arithmetic shift; absent rows sit at kFar
        const bool found = self[kind] >= 0 && res3[kind] != kNone && part < (kFar >> 1);
        const int32_t dist = part + (int32_t)cm.y;
        const int32_t other = found ? s_id[wave][(kind == 1 ? 64 : 0) + (res & 63)] : 0;
        const uint32_t code = FCODE ? ord_f32((float)dist) : ord_i32(dist);
        // a result that cannot beat the last entry of the destination list is dropped
        // (LEAN: every result goes on, k_result_csr applies the threshold)
        pass[kind] = found && (LEAN || code <= cm.x);
        entry[kind] = make_entry(code, (uint32_t)other, 3u);
        found_total += (uint32_t)__popcll(__ballot(found));
      }
    } else {
      pass[0] = pass[1] = pass[2] = false;
    }
    // slot requests for all three results first ...
    // (the two results of a NEW sample go to the same list: one request for both)
    const uint32_t want_n = (pass[0] ? 1u : 0u) + (pass[1] ? 1u : 0u);
    const uint32_t passed_total =
        (uint32_t)__popcll(__ballot(pass[0])) + (uint32_t)__popcll(__ballot(pass[1])) +
        (uint32_t)__popcll(__ballot(pass[2]));
    uint64_t word_n = 0, word_o = 0;  // direct hand-out: slot words of the destinations
    uint32_t place_n = 0, place_o = 0;  // staged hand-out: places in the buckets' LDS areas
    const int bucket_n = STAGED ? (int)((uint32_t)id_new >> sa.tb) : 0;
    const int bucket_o = STAGED ? (int)((uint32_t)id_old >> sa.tb) : 0;
    if (STAGED) {
      if (want_n) place_n = atomicAdd(&st_cnt[bucket_n], want_n);
      if (pass[2]) place_o = atomicAdd(&st_cnt[bucket_o], 1u);
      if (passed_total && lane == 0) atomicAdd(&st_fill[0], passed_total);
    } else {
      // one returning add on the destination's slot word yields the segment start
      // and the place in it
      if (want_n)
        word_n = atomicAdd(reinterpret_cast<unsigned long long*>(&pslot[id_new]),
                           (unsigned long long)want_n);
      if (pass[2])
        word_o = atomicAdd(reinterpret_cast<unsigned long long*>(&pslot[id_old]), 1ull);
    }
    // staged: places in LDS come back at once, so the results are put away before the
    // next node's rows take up the operand registers
    // (segments and bucket regions cannot overflow, see the sampling stage; the tests
    // against the array size only keep a violated bound from writing outside the array)
    if (STAGED) {
      auto put = [&](int bucket, uint32_t place, uint64_t e, int32_t dest) {
        const uint64_t rec = stage_record(e, (uint32_t)dest, sa.tb);
        if (place < (uint32_t)kStageSlots) {
          st_ent[bucket * kStageSlots + (int)place] = rec;
        } else {  // the bucket's places are taken: straight to its region
          const uint64_t at = st_region[bucket] + atomicAdd(&sa.cur[bucket], 1ull);
          if (at < slots) sa.ent[at] = rec;
          else ++over_total;
        }
      };
      if (pass[0]) put(bucket_n, place_n, entry[0], id_new);
      if (pass[1]) put(bucket_n, place_n + (pass[0] ? 1u : 0u), entry[1], id_new);
      if (pass[2]) put(bucket_o, place_o, entry[2], id_old);
    }
    // direct: with the operand registers free, the next node's rows are requested while
    // the slot words are still on their way ...
    const bool more = s1 >= 0;
    int32_t nn_new = -1, nn_old = -1;
    node_t s3 = -1;
    if (more) {
      request_rows(nx_new, nx_old);
      if (s2 >= 0 && in_list) {
        nn_new = snew[s2 * L + lane];
        nn_old = sold[s2 * L + lane];
      }
      s3 = node_at(pos + 3 * W);
    }
    // ... and only now the slots are used
    if (!STAGED) {
      const uint64_t at_n = (word_n >> kSlotCountBits) + (word_n & kSlotCountMask);
      const uint64_t at_o = (word_o >> kSlotCountBits) + (word_o & kSlotCountMask);
      if (pass[0] && pass[1]) {  // neighbouring slots: one 16-byte store
        if (at_n + 1 < slots)
          __builtin_nontemporal_store(EntryPair{entry[0], entry[1]}, reinterpret_cast<EntryPair*>(bins + at_n));
        else over_total += 2;
      } else if (want_n) {
        if (at_n < slots) __builtin_nontemporal_store(pass[0] ? entry[0] : entry[1], &bins[at_n]);
        else ++over_total;
      }
      if (pass[2]) {
        if (at_o < slots) __builtin_nontemporal_store(entry[2], &bins[at_o]);
        else ++over_total;
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) over_total += __shfl_xor(over_total, off, kWave);
    if (active && lane == 0) {
      uint64_t ev;
      if (MERGE) {
        const uint64_t cn = ((uint64_t)cls_new1 << 32) | cls_new0;
        const uint64_t co = ((uint64_t)cls_old1 << 32) | cls_old0;
        const uint64_t n1 = __popcll(cn), o1 = __popcll(co);
        ev = n1 * ((uint64_t)no - o1) + ((uint64_t)nn - n1) * o1;
      } else {
        ev = (do_nn ? (uint64_t)nn * (nn - 1) / 2 : 0) + (uint64_t)nn * no - dups;
      }
      uint64_t* cs = counters + (s & (kStripes - 1)) * C_SLOTS;
      // (k_result_csr<true>, behind a launch with a LEAN build, counts what passes the
      // thresholds)
      // (direct hand-out with a LEAN build: every result found has been handed on)
      if ((LEAN ? !STAGED : sa.count_passed) && passed_total)
        atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_PASSED),
                  (unsigned long long)passed_total);
      if (found_total) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_PROPS),
                                 (unsigned long long)found_total);
      if (over_total) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_OVERFLOW),
                                (unsigned long long)over_total);
      if (ev) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_EVALS), (unsigned long long)ev);
    }
    if (STAGED) {
      // every wave looks at the fill count after every node (a wave-uniform LDS read)
      const uint32_t fill = *reinterpret_cast<volatile uint32_t*>(st_fill);
      if ((uint32_t)__builtin_amdgcn_readfirstlane((int)fill) >= sa.threshold) (void)flush();
    }
    if (!more) break;
    pos += W;
    s = s1; s1 = s2; s2 = s3;
    id_new = nx_new; id_old = nx_old;
    nx_new = nn_new; nx_old = nn_old;
  }
  if (STAGED) {
    if (lane == 0) atomicAdd(&st_fill[1], 1u);
    while (!flush()) {
    }
  }
}

// Second half of the staged hand-out: one workgroup per bucket moves the bucket's
// results from its region into the segments of their destinations and writes the
// destinations' slot words (segment start, results received) that the list update reads.
// The results arrive in no order, and 8-byte stores to scattered places are served at a
// fixed rate whatever their number per line; so the workgroup takes the region in tiles,
// puts every tile in destination order inside LDS (counting sort: an LDS counter per
// destination gives each result its rank, a scan of the counters the start of each
// destination's run) and writes it out run by run: neighbouring lanes then store to
// neighbouring places.
constexpr int kRcBlock = 1024;
// FILTER (behind the LEAN join, which hands on every result): a result that cannot beat the
// last entry of its destination's list is dropped here, and what is left is counted as passed.
// Results per thread and tile: 12 (96 KB of LDS), 11 where the thresholds need room too.
constexpr int rc_per_thread(bool filter) { return filter ? 11 : 12; }
// LDS: the tile, then per destination of the bucket (at most 2^12) the number of results in
// the tile / the start of its run, the next free place of its segment, the segment's end
// (both relative to the region) and, with FILTER, the threshold of its list.
static size_t result_csr_lds_bytes(int tb, bool filter) {
  return (size_t)kRcBlock * rc_per_thread(filter) * 8 + (((size_t)(filter ? 4 : 3) << tb) + 1) * 4;
}

template <bool FILTER>
__global__ __launch_bounds__(kRcBlock) void k_result_csr(int64_t n, int tb,
                                                         const uint64_t* __restrict__ poff,
                                                         const unsigned long long* __restrict__ cur,
                                                         const uint64_t* __restrict__ ent,
                                                         uint64_t* __restrict__ bins,
                                                         uint64_t* __restrict__ pslot,
                                                         const NodeMeta* __restrict__ meta,
                                                         uint64_t* counters) {
  constexpr int kRcPerThread = rc_per_thread(FILTER);
  constexpr int kRcTile = kRcBlock * kRcPerThread;
  extern __shared__ __attribute__((aligned(16))) uint64_t rc_lds[];
  __shared__ uint32_t part[kRcBlock / kWave];
  uint64_t* const tile = rc_lds;
  const int T_max = 1 << tb;
  uint32_t* const run = reinterpret_cast<uint32_t*>(rc_lds + kRcTile);  // T_max + 1 entries
  uint32_t* const next = run + T_max + 1;
  uint32_t* const seg_end = next + T_max;
  uint32_t* const kth_s = seg_end + T_max;  // FILTER only
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t first = (int64_t)blockIdx.x << tb;
  const int T = (int)(n - first < (int64_t)T_max ? n - first : (int64_t)T_max);
  const uint64_t region = poff[first], room = poff[first + T] - region;
  for (int t = tid; t < T_max; t += kRcBlock) {
    next[t] = t < T ? (uint32_t)(poff[first + t] - region) : (uint32_t)room;
    seg_end[t] = t < T ? (uint32_t)(poff[first + t + 1] - region) : (uint32_t)room;
    if (FILTER) kth_s[t] = t < T ? meta[first + t].kth : 0u;
  }
  uint32_t kept = 0;  // FILTER: results that pass
  uint64_t count = cur[blockIdx.x];
  if (count > room) {  // cannot happen: a region holds what its destinations can receive
    if (tid == 0)
      atomicAdd(reinterpret_cast<unsigned long long*>(counters + C_OVERFLOW),
                (unsigned long long)(count - room));
    count = room;
  }
  const int per = (T_max + kRcBlock - 1) / kRcBlock;  // counters per thread in the scan (<= 4)
  for (uint64_t base = 0; base < count; base += kRcTile) {
    for (int t = tid; t <= T_max; t += kRcBlock) run[t] = 0;
    __syncthreads();
    // rank of every result among the tile's results for the same destination
    uint64_t e[kRcPerThread];
    uint32_t rank[kRcPerThread];
#pragma unroll
    for (int r = 0; r < kRcPerThread; ++r) {
      const uint64_t i = base + (uint64_t)r * kRcBlock + tid;
      e[r] = i < count ? ent[region + i] : ~0ull;
    }
#pragma unroll
    for (int r = 0; r < kRcPerThread; ++r) {
      const int t = (int)(((uint32_t)e[r] >> kStageIdBits) & (uint32_t)(T_max - 1));
      if (e[r] == ~0ull || t >= T || (FILTER && (uint32_t)(e[r] >> 32) > kth_s[t])) {
        e[r] = ~0ull;
      } else {
        rank[r] = atomicAdd(&run[t], 1u);
        ++kept;
      }
    }
    __syncthreads();
    // exclusive scan of the counters: thread i takes counters per*i .. per*i + per - 1
    uint32_t mine[4], sum = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int t = tid * per + j;
      mine[j] = (j < per && t < T_max) ? run[t] : 0u;
      sum += mine[j];
    }
    uint32_t inc = sum;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const uint32_t o = __shfl_up(inc, off, kWave);
      if (lane >= off) inc += o;
    }
    if (lane == kWave - 1) part[wave] = inc;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += part[w];
    uint32_t at = before + inc - sum;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int t = tid * per + j;
      if (j < per && t < T_max) run[t] = at;
      at += mine[j];
    }
    if (tid == kRcBlock - 1) run[T_max] = at;  // results in the tile
    __syncthreads();
    // the tile in destination order
#pragma unroll
    for (int r = 0; r < kRcPerThread; ++r) {
      if (e[r] != ~0ull) {
        const int t = (int)(((uint32_t)e[r] >> kStageIdBits) & (uint32_t)(T_max - 1));
        tile[run[t] + rank[r]] = e[r];
      }
    }
    __syncthreads();
    const uint32_t in_tile = run[T_max];
#pragma unroll
    for (int r = 0; r < kRcPerThread; ++r) {
      const uint32_t j = (uint32_t)r * kRcBlock + tid;
      if (j < in_tile) {
        const uint64_t x = tile[j];
        const int t = (int)(((uint32_t)x >> kStageIdBits) & (uint32_t)(T_max - 1));
        const uint32_t place = next[t] + (j - run[t]);
        // back to a list entry: distance code | object id | "admitted now" + NEW
        if (place < seg_end[t])
          bins[region + place] = make_entry((uint32_t)(x >> 32),
                                            (uint32_t)x & ((1u << kStageIdBits) - 1u), 3u);
      }
    }
    __syncthreads();
    for (int t = tid; t < T; t += kRcBlock) next[t] += run[t + 1] - run[t];
    __syncthreads();
  }
  __syncthreads();
  if (FILTER) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) kept += __shfl_xor(kept, off, kWave);
    if (lane == 0 && kept)
      atomicAdd(reinterpret_cast<unsigned long long*>(
                    counters +
                    ((blockIdx.x * (kRcBlock / kWave) + wave) & (kStripes - 1)) * C_SLOTS + C_PASSED),
                (unsigned long long)kept);
  }
  for (int t = tid; t < T; t += kRcBlock) {
    const uint64_t start = poff[first + t] - region;
    const uint64_t end = next[t] < seg_end[t] ? next[t] : seg_end[t];
    const uint64_t got = end - start < kSlotCountMask ? end - start : kSlotCountMask;
    pslot[first + t] = ((region + start) << kSlotCountBits) | got;
  }
}

// The nodes that have something to evaluate, listed by shape (list c at nodes + c n, its
// length in count[c]; the order inside a list is of no consequence).  A workgroup takes
// kShapeNodes consecutive nodes, numbers those of each list in LDS and reserves their places
// with one addition per list.
constexpr int kShapePerThread = 16;
constexpr int kShapeNodes = 256 * kShapePerThread;
__global__ __launch_bounds__(256) void k_join_shapes(int64_t n, int merge_mode,
                                                     const int32_t* __restrict__ cnew,
                                                     const int32_t* __restrict__ cold,
                                                     int32_t* nodes, uint32_t* count) {
  __shared__ uint32_t here[kJoinShapes], base[kJoinShapes];
  const int64_t first = block_linear() * kShapeNodes;
  if (threadIdx.x < kJoinShapes) here[threadIdx.x] = 0u;
  __syncthreads();
  int32_t place[kShapePerThread];  // list + kJoinShapes x (number within the workgroup)
#pragma unroll
  for (int j = 0; j < kShapePerThread; ++j) {
    const int64_t s = first + j * 256 + threadIdx.x;
    place[j] = -1;
    if (s < n) {
      const int nn = cnew[s], no = cold[s];
      const bool do_nn = !merge_mode && nn > 1;
      if (nn > 0 && (do_nn || no > 0)) {
        const int c = join_list_of_shape(no <= 32 ? 1 : nn <= 32 ? 2 : 0);
        place[j] = c + kJoinShapes * (int32_t)atomicAdd(&here[c], 1u);
      }
    }
  }
  __syncthreads();
  if (threadIdx.x < kJoinShapes && here[threadIdx.x] != 0u)
    base[threadIdx.x] = atomicAdd(&count[threadIdx.x], here[threadIdx.x]);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kShapePerThread; ++j) {
    if (place[j] >= 0) {
      const int c = place[j] % kJoinShapes;
      nodes[(int64_t)c * n + base[c] + place[j] / kJoinShapes] =
          (int32_t)(first + j * 256 + threadIdx.x);
    }
  }
}

template <int KSTEPS, bool STAGED, bool LEAN = false, int SHAPE = 0>
static hipError_t launch_k(bool fcode, bool merge, unsigned grid, hipStream_t st,
                           const int8_t* shadow, const NodeMeta* meta, int dpad, const Shape& sh,
                           const DevState& ds, const StageArgs& sa) {
  constexpr int block = join_waves(STAGED, SHAPE) * kWave;
  const size_t lds = STAGED ? kStageLdsBytes : 0;
#define GNND_ARGS shadow, meta, dpad, sh.n, sh.p, sh.split, ds.snew, ds.sold, \
                  ds.pslot, (uint64_t)sh.slots(), ds.bins, ds.counters, sa
#define GNND_LAUNCH(F, M)                                                                      \
  do {                                                                                         \
    auto* kern = k_join_mfma<KSTEPS, F, M, STAGED, LEAN, SHAPE>;                               \
    if (STAGED) {                                                                              \
      static bool attr_set = false; /* per instantiation: a staging area beyond the default */ \
      if (!attr_set) {                                                                         \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                \
                                           hipFuncAttributeMaxDynamicSharedMemorySize,         \
                                           (int)kStageLdsBytes);                               \
        if (e != hipSuccess) return e;                                                         \
        attr_set = true;                                                                       \
      }                                                                                        \
    }                                                                                          \
    kern<<<grid, block, lds, st>>>(GNND_ARGS);                                                 \
  } while (0)
  if (LEAN) {  // never with a merge
    if (fcode) GNND_LAUNCH(true, false);
    else GNND_LAUNCH(false, false);
  } else if (fcode) {
    if (merge) GNND_LAUNCH(true, true);
    else GNND_LAUNCH(true, false);
  } else {
    if (merge) GNND_LAUNCH(false, true);
    else GNND_LAUNCH(false, false);
  }
#undef GNND_LAUNCH
#undef GNND_ARGS
  return hipGetLastError();
}

static int compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cus = v;
    else
      cus = 256;
  }
  return cus;
}

hipError_t launch_join_mfma(const Shape& sh, const DevState& ds, bool merge_mode, bool first_look,
                            hipStream_t st, hipEvent_t after_join) {
  const int dpad = (sh.d + 31) & ~31;
  const int ksteps = dpad / 32;
  const bool fcode = sh.metric != kL2U8;
  const bool staged = ds.stg_ent != nullptr;
  // the first iteration on a random graph: see LEAN
  const bool lean = first_look && !merge_mode;
  StageArgs sa{ds.stg_ent, ds.stg_cur, ds.poff, 0, 0, 0, ds.cls_nodes, ds.cls_count, !(lean && staged)};
  hipError_t e;
  if (!staged) {
    // persistent wavefronts: about two resident sets of workgroups, each wave strides over nodes
    const int64_t want = (sh.n + 3) / 4;
    const unsigned grid = (unsigned)(want < kJoinGrid ? want : kJoinGrid);
#define GNND_K(K)                                                                               \
  e = lean ? launch_k<K, false, true>(fcode, false, grid, st, ds.shadow, ds.meta, dpad, sh, ds, sa) \
           : launch_k<K, false>(fcode, merge_mode, grid, st, ds.shadow, ds.meta, dpad, sh, ds, sa)
    switch (ksteps) {
      case 1: GNND_K(1); break;
      case 2: GNND_K(2); break;
      case 3: GNND_K(3); break;
      default: GNND_K(4);
    }
#undef GNND_K
    if (after_join) (void)hipEventRecord(after_join, st);
    return e;
  }
  sa.tb = stage_bucket_bits(sh.n);
  sa.nb = (int)((sh.n + ((int64_t)1 << sa.tb) - 1) >> sa.tb);
  // flush at half-full on average: few results find their bucket's places taken
  sa.threshold = (uint32_t)(sa.nb * (kStageSlots / 2));
  e = launch_zero_u32(reinterpret_cast<uint32_t*>(ds.stg_cur), 2 * kStageBuckets, st);
  if (e == hipSuccess) e = launch_zero_u32(ds.cls_count, kJoinShapes, st);
  if (e != hipSuccess) return e;
  k_join_shapes<<<grid_blocks((sh.n + kShapeNodes - 1) / kShapeNodes), 256, 0, st>>>(
      sh.n, merge_mode ? 1 : 0, ds.cnew, ds.cold, ds.cls_nodes, ds.cls_count);
  // persistent workgroups, one per CU (the staging area takes most of a CU's LDS); one launch
  // per shape, the common shapes first; all of them add to the same bucket regions
  auto grid_for = [&](int waves) {
    const int64_t want = (sh.n + waves - 1) / waves;
    return (unsigned)(want < compute_units() ? want : compute_units());
  };
  const unsigned grid_slim = grid_for(kStagedWavesSlim), grid_full = grid_for(kStagedWaves);
#define GNND_K(K)                                                                                  \
  e = lean ? launch_k<K, true, true, 1>(fcode, false, grid_slim, st, ds.shadow, ds.meta, dpad, sh, \
                                        ds, sa)                                                    \
           : launch_k<K, true, false, 1>(fcode, merge_mode, grid_slim, st, ds.shadow, ds.meta,     \
                                         dpad, sh, ds, sa);                                        \
  if (e == hipSuccess)                                                                             \
    e = launch_k<K, true, false, 2>(fcode, merge_mode, grid_slim, st, ds.shadow, ds.meta, dpad,    \
                                    sh, ds, sa);                                                   \
  if (e == hipSuccess)                                                                             \
    e = launch_k<K, true, false, 0>(fcode, merge_mode, grid_full, st, ds.shadow, ds.meta, dpad,    \
                                    sh, ds, sa)
  switch (ksteps) {
    case 1: GNND_K(1); break;
    case 2: GNND_K(2); break;
    case 3: GNND_K(3); break;
    default: GNND_K(4);
  }
#undef GNND_K
  if (after_join) (void)hipEventRecord(after_join, st);
  if (e != hipSuccess) return e;
  // (a region is shorter than 2^32 slots: n <= 2^20, 6p <= 192 slots per node)
  const size_t lds = result_csr_lds_bytes(sa.tb, lean);
  auto* csr = lean ? &k_result_csr<true> : &k_result_csr<false>;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(csr),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  csr<<<(unsigned)sa.nb, kRcBlock, lds, st>>>(sh.n, sa.tb, ds.poff, ds.stg_cur, ds.stg_ent, ds.bins,
                                             ds.pslot, ds.meta, ds.counters);
  return hipGetLastError();
}

hipError_t launch_init_random_i8(const Shape& sh, const DevState& ds, uint64_t seed,
                                 hipStream_t st) {
  // long or segmented lists: the general kernels on the original vectors give the same integers
  if (sh.segments > 1) return launch_init_random_segmented(sh, ds, seed, st);
  if (sh.k > kWave) return launch_init_random_wide(sh, ds, seed, st);
  const int dpad = (sh.d + 31) & ~31;
  const dim3 grid = grid_blocks((sh.n + 3) / 4);
  const uint64_t base = hash_base(seed, kTagInit);
  if (sh.metric != kL2U8)
    k_init_random_i8<true><<<grid, 256, 0, st>>>(ds.shadow, ds.meta, dpad, sh.n, sh.k, base, ds.G);
  else
    k_init_random_i8<false><<<grid, 256, 0, st>>>(ds.shadow, ds.meta, dpad, sh.n, sh.k, base, ds.G);
  return hipGetLastError();
}

hipError_t launch_merge_init_i8(const Shape& sh, const DevState& ds, uint64_t seed,
                                const MergeIds& mi, const int32_t* ids1, const void* dist1,
                                const int32_t* ids2, const void* dist2, hipStream_t st) {
  // long lists: the general kernel on the original vectors gives the same integers
  if (sh.k > kWave) return launch_merge_init(sh, ds, seed, mi, ids1, dist1, ids2, dist2, st);
  const int dpad = (sh.d + 31) & ~31;
  const dim3 grid = grid_blocks((sh.n + 3) / 4);
  const uint64_t base = hash_base(seed, kTagMerge);
  if (sh.metric != kL2U8)
    k_merge_init_i8<true><<<grid, 256, 0, st>>>(ds.shadow, ds.meta, dpad, sh.n, mi, sh.k, base, ids1,
                                                dist1, ids2, dist2, ds.G, ds.aside);
  else
    k_merge_init_i8<false><<<grid, 256, 0, st>>>(ds.shadow, ds.meta, dpad, sh.n, mi, sh.k, base,
                                                 ids1, dist1, ids2, dist2, ds.G, ds.aside);
  return hipGetLastError();
}

hipError_t launch_pack_i8(const Shape& sh, const DevState& ds, int* bad_flag_dev,
                          hipStream_t st) {
  const int dpad = (sh.d + 31) & ~31;
  const dim3 grid = grid_blocks((sh.n + 3) / 4);
  if (sh.metric == kL2U8 && (sh.d & 15) == 0) {
    const int64_t per_block = 4 * (kWave / (dpad >> 4));  // rows per workgroup
    k_pack_u8_wide<<<grid_blocks((sh.n + per_block - 1) / per_block), 256, 0, st>>>(
        static_cast<const uint8_t*>(sh.vec_a), static_cast<const uint8_t*>(sh.vec_b), sh.split,
        sh.n, sh.d, dpad, ds.shadow, ds.meta);
  } else if (sh.metric == kL2U8)
    k_pack_i8<uint8_t><<<grid, 256, 0, st>>>(sh.vec_a, sh.vec_b, sh.split, sh.n, sh.d, dpad,
                                             ds.shadow, ds.meta, bad_flag_dev);
  else
    k_pack_i8<float><<<grid, 256, 0, st>>>(sh.vec_a, sh.vec_b, sh.split, sh.n, sh.d, dpad,
                                           ds.shadow, ds.meta, bad_flag_dev);
  return hipGetLastError();
}

}  // namespace gnnd
