// Lists of 65..128 entries (the paper's runs with k up to 128, Sec. 6.3): the
// graph-side kernels again give one wavefront to a list, which now holds two
// entries per lane - entry i sits in lane i % 64 of register i / 64.  Sorting is
// two 64-lane networks plus a 128-wide bitonic merge; a sorted chunk of 64
// candidates is merged into the list by splitting (smaller half / larger half)
// against the first register and merging the larger half into the second
// (sort128 / merge128).  The length of the sample lists is another matter (2p).
#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

namespace {

constexpr int kWB = 256;
constexpr int kWavesPerWB = kWB / kWave;

__device__ inline int64_t wide_wave_index() {
  return block_linear() * kWavesPerWB + wave_id();
}
inline dim3 wide_blocks(int64_t waves) {
  return grid_blocks((waves + kWavesPerWB - 1) / kWavesPerWB);
}

// lower bound of key kk among the 64 ascending entries of `row`, compared on (distance, id)
__device__ inline bool holds_key(uint64_t row, uint64_t kk) {
  int pos = 0;
#pragma unroll
  for (int step = kWave / 2; step > 0; step >>= 1) {
    const uint64_t r = __shfl(row, pos + step - 1, kWave);
    pos += (entry_key(r) < kk) ? step : 0;
  }
  return entry_key(__shfl(row, pos, kWave)) == kk;
}

// The wide form of the candidate filter of the update: drop what is not closer
// than the list's last entry, what the list already holds, and repeats; the
// survivors come back ascending.
__device__ inline uint64_t filter_candidates_wide(uint64_t pk, uint64_t lo, uint64_t hi, int k,
                                                  int lane, bool& any) {
  const uint64_t last = readlane64(hi, k - 1 - kWave);
  if (pk != kKeyMax && entry_key(pk) >= entry_key(last)) pk = kKeyMax;
  any = __ballot(pk != kKeyMax) != 0ull;
  if (!any) return pk;
  const uint64_t kk = entry_key(pk);
  // both searches by all lanes: they read each other's registers
  const bool in_lo = holds_key(lo, kk);
  const bool in_hi = holds_key(hi, kk);
  if (in_lo || in_hi) pk = kKeyMax;
  const uint64_t left = __ballot(pk != kKeyMax);
  any = left != 0ull;
  if (!any) return pk;
  pk = wave_compact(pk, pk != kKeyMax, kKeyMax, lane);
  pk = wave_sort_upto(pk, lane, __popcll(left));
  const uint64_t prev = __shfl_up(pk, 1, kWave);
  const bool rep = lane > 0 && pk != kKeyMax && entry_key(pk) == entry_key(prev);
  if (__ballot(rep) != 0ull) pk = wave_compact(pk, !rep, kKeyMax, lane);
  return pk;
}

// `count` (65..128) distinct ids, two slots per lane (slot lane and slot lane +
// 64), by the same slot-by-slot rule as draw_distinct.
__device__ inline void draw_distinct_wide(uint64_t base_hash, uint32_t s, int count, uint32_t range,
                                          uint32_t base, uint32_t forbid, int lane, uint32_t& out0,
                                          uint32_t& out1) {
  const bool have1 = lane + kWave < count;
  const uint32_t f0 = bounded(hash3(base_hash, s, (uint32_t)lane, 0u), range) + base;
  const uint32_t f1 = bounded(hash3(base_hash, s, (uint32_t)(lane + kWave), 0u), range) + base;
  bool clash_any = f0 == forbid || (have1 && f1 == forbid);
  for (int j = 0; j + 1 < count; ++j) {
    const uint32_t cj = j < kWave ? (uint32_t)__builtin_amdgcn_readlane((int)f0, j)
                                  : (uint32_t)__builtin_amdgcn_readlane((int)f1, j - kWave);
    clash_any |= (lane > j && f0 == cj) || (have1 && lane + kWave > j && f1 == cj);
  }
  if (__ballot(clash_any) == 0ull) {
    out0 = f0;
    out1 = f1;
    return;
  }
  uint32_t m0 = 0xffffffffu, m1 = 0xffffffffu;
  for (int j = 0; j < count; ++j) {
    uint32_t cand = 0;
    bool ok = false;
    for (uint32_t attempt = 0; attempt < kHashAttempts && !ok; ++attempt) {
      cand = bounded(hash3(base_hash, s, (uint32_t)j, attempt), range) + base;
      const bool clash = (lane < j && m0 == cand) || (lane + kWave < j && m1 == cand);
      ok = (cand != forbid) && (__ballot(clash) == 0ull);
    }
    for (uint32_t step = 0; step < range && !ok; ++step) {
      uint32_t local = cand - base;
      local = (local + 1 == range) ? 0 : local + 1;
      cand = local + base;
      const bool clash = (lane < j && m0 == cand) || (lane + kWave < j && m1 == cand);
      ok = (cand != forbid) && (__ballot(clash) == 0ull);
    }
    if (lane == j) m0 = cand;
    if (lane + kWave == j) m1 = cand;
  }
  out0 = m0;
  out1 = m1;
}

// ---------------------------------------------------------------------------
// Alg. 1, first loop, for 64 < k <= 128.
template <int METRIC>
__global__ __launch_bounds__(kWB) void k_init_random_wide(VecSrc vs, int64_t n, int k,
                                                          uint64_t base_hash, uint64_t* G,
                                                          NodeMeta* meta) {
  __shared__ uint32_t tile[kWavesPerWB][kEvalTileWords];
  const int64_t s = wide_wave_index();
  if (s >= n) return;
  const int lane = lane_id();
  uint32_t id0, id1;
  draw_distinct_wide(base_hash, (uint32_t)s, k, (uint32_t)n, 0u, (uint32_t)s, lane, id0, id1);
  uint32_t* my_tile = tile[wave_id()];
  const uint32_t c0 = wave_distances<METRIC>(vs, (uint32_t)s, id0, true, my_tile, lane);
  const uint32_t c1 = wave_distances<METRIC>(vs, (uint32_t)s, id1, lane + kWave < k, my_tile, lane);
  uint64_t lo = make_entry(c0, id0, 1u);
  uint64_t hi = lane + kWave < k ? make_entry(c1, id1, 1u) : kKeyMax;
  sort128(lo, hi, lane);
  G[s * k + lane] = lo;
  if (lane + kWave < k) G[s * k + kWave + lane] = hi;
  if (lane + kWave == k - 1) meta[s].kth = entry_code(hi);
}

// ---------------------------------------------------------------------------
// Sec. 4.3 list insertion, all proposals of one destination at once, 64 < k <= 128.
__global__ __launch_bounds__(kWB) void k_update_wide(int64_t n, int k, uint64_t* G, NodeMeta* meta,
                                                     const uint64_t* pslot, const uint64_t* poff,
                                                     const uint64_t* bins, uint64_t* counters) {
  const int64_t u = wide_wave_index();
  if (u >= n) return;
  const int lane = lane_id();
  uint64_t cnt = pslot[u] & kSlotCountMask;
  const uint64_t beg = poff[u], cap = poff[u + 1] - beg;
  uint64_t lo = G[u * k + lane];
  uint64_t hi = lane + kWave < k ? G[u * k + kWave + lane] : kKeyMax;
  if (cnt == 0) return;
  uint64_t* cs = counters + (u & (kStripes - 1)) * C_SLOTS;
  if (cnt > cap) {  // cannot happen: a segment is sized by the bound of what its node can receive
    if (lane == 0)
      atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_OVERFLOW), (unsigned long long)(cnt - cap));
    cnt = cap;
  }
  bool changed = false;
  for (uint64_t c = 0; c < cnt; c += kWave) {
    uint64_t pk = (c + lane < cnt) ? bins[beg + c + lane] : kKeyMax;
    bool any;
    pk = filter_candidates_wide(pk, lo, hi, k, lane, any);
    if (!any) continue;
    merge128(lo, hi, pk, lane);
    if (lane + kWave >= k) hi = kKeyMax;
    changed = true;
  }
  if (!changed) return;
  const uint64_t adm0 = __ballot((lo & 2ull) != 0);
  const uint64_t adm1 = __ballot(lane + kWave < k && (hi & 2ull) != 0);
  G[u * k + lane] = lo & ~2ull;
  if (lane + kWave < k) G[u * k + kWave + lane] = hi & ~2ull;
  if (lane + kWave == k - 1) meta[u].kth = entry_code(hi);
  if (lane == 0)
    atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_INSERTS),
              (unsigned long long)(__popcll(adm0) + __popcll(adm1)));
}

// ---------------------------------------------------------------------------
// GGM, Alg. 3 "Divide" + "Append" for 64 < k <= 128: the first ceil(k/2) <= 64
// entries stay (OLD), the rest is set aside, floor(k/2) <= 64 random objects of
// the other set come in (NEW); the (distance, id) order is restored.
template <int METRIC>
__global__ __launch_bounds__(kWB) void k_merge_init_wide(VecSrc vs, int64_t n, MergeIds mi, int k,
                                                         uint64_t base_hash, const int32_t* ids1,
                                                         const void* dist1, const int32_t* ids2,
                                                         const void* dist2, uint64_t* G,
                                                         NodeMeta* meta, uint64_t* aside) {
  __shared__ uint32_t tile[kWavesPerWB][kEvalTileWords];
  const int64_t s = wide_wave_index();
  if (s >= n) return;
  const int lane = lane_id();
  const int64_t n1 = mi.n1;
  const bool first = s < n1;
  const int64_t loc = first ? s : s - n1;
  const int32_t* sid = (first ? ids1 : ids2) + loc * k;
  const void* sdist = first ? dist1 : dist2;
  const int keep = (k + 1) / 2, fill = k / 2;
  auto load = [&](int i) {  // entry i of the input list, renumbered for this merge, flagged OLD
    const uint32_t id = mi.to_internal(sid[i]);
    const uint32_t code = METRIC == kL2U8
                              ? ord_i32(reinterpret_cast<const int32_t*>(sdist)[loc * k + i])
                              : ord_f32(reinterpret_cast<const float*>(sdist)[loc * k + i]);
    return make_entry(code, id, 0u);
  };
  const uint64_t in0 = load(lane);
  const uint64_t in1 = lane + kWave < k ? load(lane + kWave) : kKeyMax;
  if (lane >= keep) aside[s * fill + (lane - keep)] = in0;
  if (lane + kWave < k) aside[s * fill + (lane + kWave - keep)] = in1;
  const uint32_t draw = draw_distinct(base_hash, (uint32_t)s, fill,
                                      (uint32_t)(first ? n - n1 : n1), first ? (uint32_t)n1 : 0u,
                                      0xffffffffu, lane);
  uint64_t lo = lane < keep ? in0 : kKeyMax;
  const uint32_t cd =
      wave_distances<METRIC>(vs, (uint32_t)s, draw, lane < fill, tile[wave_id()], lane);
  uint64_t hi = lane < fill ? make_entry(cd, draw, 1u) : kKeyMax;
  sort128(lo, hi, lane);
  G[s * k + lane] = lo;
  if (lane + kWave < k) G[s * k + kWave + lane] = hi;
  if (lane + kWave == k - 1) meta[s].kth = entry_code(hi);
}

// GGM, Alg. 3 "Merge and Sort" for 64 < k <= 128.
template <bool FLOAT>
__global__ __launch_bounds__(kWB) void k_merge_final_wide(int64_t n, MergeIds mi, int k,
                                                          const uint64_t* G, const uint64_t* aside,
                                                          int32_t* ids_out, void* dist_out) {
  const int64_t s = wide_wave_index();
  if (s >= n) return;
  const int lane = lane_id();
  const int fill = k / 2;
  uint64_t lo = G[s * k + lane];
  uint64_t hi = lane + kWave < k ? G[s * k + kWave + lane] : kKeyMax;
  uint64_t pk = lane < fill ? aside[s * fill + lane] : kKeyMax;
  bool any;
  pk = filter_candidates_wide(pk, lo, hi, k, lane, any);
  if (any) {
    merge128(lo, hi, pk, lane);
    if (lane + kWave >= k) hi = kKeyMax;
  }
  // renumber, then restore the order under the new ids (only ties can move)
  lo = make_entry(entry_code(lo), (uint32_t)mi.to_global(entry_id(lo)), 0u);
  hi = lane + kWave < k ? make_entry(entry_code(hi), (uint32_t)mi.to_global(entry_id(hi)), 0u)
                        : kKeyMax;
  sort128(lo, hi, lane);
  auto store = [&](int i, uint64_t e) {
    ids_out[s * k + i] = (int32_t)entry_id(e);
    if (FLOAT) reinterpret_cast<float*>(dist_out)[s * k + i] = unord_f32(entry_code(e));
    else reinterpret_cast<int32_t*>(dist_out)[s * k + i] = unord_i32(entry_code(e));
  };
  store(lane, lo);
  if (lane + kWave < k) store(lane + kWave, hi);
}

VecSrc wide_vec_src(const Shape& sh) {
  return VecSrc{sh.vec_a, sh.vec_b, sh.split, sh.d, sh.norms};
}

}  // namespace

hipError_t launch_init_random_wide(const Shape& sh, const DevState& ds, uint64_t seed,
                                   hipStream_t st) {
  const dim3 grid = wide_blocks(sh.n);
  const uint64_t base = hash_base(seed, kTagInit);
  switch (sh.metric) {
    case kL2F32:
      k_init_random_wide<kL2F32><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, sh.k, base, ds.G,
                                                       ds.meta);
      break;
    case kAngularF32:
      k_init_random_wide<kAngularF32><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, sh.k, base,
                                                            ds.G, ds.meta);
      break;
    case kChi2F32:
      k_init_random_wide<kChi2F32><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, sh.k, base, ds.G,
                                                         ds.meta);
      break;
    case kCosineF32:
      k_init_random_wide<kCosineF32><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, sh.k, base,
                                                           ds.G, ds.meta);
      break;
    default:
      k_init_random_wide<kL2U8><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, sh.k, base, ds.G,
                                                      ds.meta);
  }
  return hipGetLastError();
}

hipError_t launch_update_wide(const Shape& sh, const DevState& ds, hipStream_t st) {
  k_update_wide<<<wide_blocks(sh.n), kWB, 0, st>>>(sh.n, sh.k, ds.G, ds.meta, ds.pslot, ds.poff,
                                                   ds.bins, ds.counters);
  return hipGetLastError();
}

hipError_t launch_merge_init_wide(const Shape& sh, const DevState& ds, uint64_t seed,
                                  const MergeIds& mi, const int32_t* ids1, const void* dist1,
                                  const int32_t* ids2, const void* dist2, hipStream_t st) {
  const dim3 grid = wide_blocks(sh.n);
  const uint64_t base = hash_base(seed, kTagMerge);
  switch (sh.metric) {
    case kL2F32:
      k_merge_init_wide<kL2F32><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, mi, sh.k, base, ids1,
                                                      dist1, ids2, dist2, ds.G, ds.meta, ds.aside);
      break;
    case kAngularF32:
      k_merge_init_wide<kAngularF32><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, mi, sh.k, base,
                                                           ids1, dist1, ids2, dist2, ds.G, ds.meta,
                                                           ds.aside);
      break;
    case kChi2F32:
      k_merge_init_wide<kChi2F32><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, mi, sh.k, base,
                                                        ids1, dist1, ids2, dist2, ds.G, ds.meta,
                                                        ds.aside);
      break;
    case kCosineF32:
      k_merge_init_wide<kCosineF32><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, mi, sh.k, base,
                                                          ids1, dist1, ids2, dist2, ds.G, ds.meta,
                                                          ds.aside);
      break;
    default:
      k_merge_init_wide<kL2U8><<<grid, kWB, 0, st>>>(wide_vec_src(sh), sh.n, mi, sh.k, base, ids1,
                                                     dist1, ids2, dist2, ds.G, ds.meta, ds.aside);
  }
  return hipGetLastError();
}

hipError_t launch_merge_final_wide(const Shape& sh, const DevState& ds, const MergeIds& mi,
                                   int32_t* ids_out, void* dist_out, hipStream_t st) {
  const dim3 grid = wide_blocks(sh.n);
  if (sh.metric == kL2U8)
    k_merge_final_wide<false><<<grid, kWB, 0, st>>>(sh.n, mi, sh.k, ds.G, ds.aside, ids_out,
                                                    dist_out);
  else
    k_merge_final_wide<true><<<grid, kWB, 0, st>>>(sh.n, mi, sh.k, ds.G, ds.aside, ids_out,
                                                   dist_out);
  return hipGetLastError();
}

}  // namespace gnnd
