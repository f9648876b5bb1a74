// Segmented k-NN lists (Sec. 4.3, "Multiple Spinlocks"): a list of k = 32 m
// entries (k = 64, 96, 128) is m segments of 32, object v can only live in
// segment v % m, and when an iteration is over the segments are merged into one
// ascending list.  The paper guards each segment with a spinlock of its own and
// gives it one warp of 32; here one 64-lane wavefront owns the whole list, holds
// every segment in the lower half of a register, inserts all proposals of a class
// into its segment at once (best 32 of segment and proposals, by (distance, id):
// what the locked insertions give in any order) and merges the segments at the
// end.  Between iterations the rows are stored merged, as every other kernel
// expects them.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

namespace {

constexpr int kSGB = 256;
constexpr int kWavesPerSGB = kSGB / kWave;
constexpr int kSeg = 32;        // entries per segment
constexpr int kMaxSegments = 4; // k <= 128

__device__ inline int64_t seg_wave_index() {
  return block_linear() * kWavesPerSGB + wave_id();
}
inline dim3 seg_blocks(int64_t waves) {
  return grid_blocks((waves + kWavesPerSGB - 1) / kWavesPerSGB);
}

// Entry i of the list as drawn sits in lane i % 64 of register i / 64: its segment is
// r = i / 32, its slot inside the segment j = i % 32.
//
// Alg. 1, first loop, for a segmented list: every segment gets 32 distinct random
// members of its residue class other than the node itself.  Slot 32 r + j takes member
// number hash(seed, INIT, s, 32 r + j, attempt) mapped onto the class size for attempt =
// 0, 1, ... until it differs from the node and from the earlier slots of its segment;
// after kHashAttempts failures it walks to the next free member cyclically.
template <int METRIC>
__global__ __launch_bounds__(kSGB) void k_init_random_segmented(VecSrc vs, int64_t n, int k,
                                                                uint64_t base_hash, uint64_t* G,
                                                                NodeMeta* meta) {
  __shared__ uint32_t tile[kWavesPerSGB][kEvalTileWords];
  const int64_t s = seg_wave_index();
  if (s >= n) return;
  const int lane = lane_id();
  const int m = k / kSeg;
  const int j = lane & (kSeg - 1);
  const uint64_t group = 0xffffffffull << (lane & kSeg);  // the 32 lanes of this lane's segment
  uint32_t members[2], own[2], local[2];
  bool on[2];
#pragma unroll
  for (int reg = 0; reg < 2; ++reg) {
    const int r = (lane >> 5) + 2 * reg;
    on[reg] = r < m;
    members[reg] = on[reg] ? (uint32_t)((n - r + m - 1) / m) : 1u;  // ids r, r + m, r + 2m, ...
    own[reg] = (on[reg] && (int)(s % m) == r) ? (uint32_t)(s / m) : 0xffffffffu;
    local[reg] = bounded(hash3(base_hash, (uint32_t)s, (uint32_t)(kSeg * r + j), 0u), members[reg]);
  }
  // Are the first attempts valid as they stand (distinct inside every segment, none the
  // node itself)?  Then the slot-by-slot rule accepts every one of them.
  bool clash = (on[0] && local[0] == own[0]) || (on[1] && local[1] == own[1]);
  for (int t = 0; t + 1 < kSeg; ++t) {
    const int src = (lane & kSeg) | t;
    const uint32_t o0 = __shfl(local[0], src, kWave), o1 = __shfl(local[1], src, kWave);
    clash |= t < j && ((on[0] && o0 == local[0]) || (on[1] && o1 == local[1]));
  }
  if (__ballot(clash) != 0ull) {
    uint32_t mine[2] = {0xffffffffu, 0xffffffffu};
    for (int slot = 0; slot < kSeg; ++slot) {
      // every lane of a segment computes the segment's candidate for this slot
      uint32_t cand[2] = {0, 0}, attempt[2] = {0, 0}, steps[2] = {0, 0};
      bool ok[2] = {!on[0], !on[1]};
      while (__ballot(!ok[0] || !ok[1]) != 0ull) {
#pragma unroll
        for (int reg = 0; reg < 2; ++reg) {
          const int r = (lane >> 5) + 2 * reg;
          if (!ok[reg]) {
            if (attempt[reg] < kHashAttempts) {
              cand[reg] = bounded(hash3(base_hash, (uint32_t)s, (uint32_t)(kSeg * r + slot),
                                        attempt[reg]), members[reg]);
              ++attempt[reg];
            } else {  // at most `members` steps: the host has checked that enough ids are free
              cand[reg] = cand[reg] + 1 == members[reg] ? 0u : cand[reg] + 1;
              ++steps[reg];
            }
          }
          const bool taken = !ok[reg] && j < slot && mine[reg] == cand[reg];
          const bool group_taken = (__ballot(taken) & group) != 0ull;
          if (!ok[reg])
            ok[reg] = (cand[reg] != own[reg] && !group_taken) || steps[reg] > members[reg];
        }
      }
      if (j == slot) {
        mine[0] = cand[0];
        mine[1] = cand[1];
      }
    }
    local[0] = mine[0];
    local[1] = mine[1];
  }
  uint64_t e[2];
#pragma unroll
  for (int reg = 0; reg < 2; ++reg) {
    const int r = (lane >> 5) + 2 * reg;
    const uint32_t id = on[reg] ? local[reg] * (uint32_t)m + (uint32_t)r : 0u;
    e[reg] = kKeyMax;
    if (reg == 0 || k > kWave) {  // uniform
      const uint32_t code =
          wave_distances<METRIC>(vs, (uint32_t)s, id, on[reg], tile[wave_id()], lane);
      if (on[reg]) e[reg] = make_entry(code, id, 1u);
    }
  }
  sort128(e[0], e[1], lane);
  G[s * k + lane] = e[0];
  if (lane + kWave < k) G[s * k + kWave + lane] = e[1];
  const int last = k - 1;
  if (lane == (last & 63)) meta[s].kth = entry_code(last < kWave ? e[0] : e[1]);
}

// Sec. 4.3 list insertion for all proposals of one destination at once, into its
// segments: a proposal for object v competes with segment v % m only.
__global__ __launch_bounds__(kSGB) void k_update_segmented(int64_t n, int k, uint64_t* G,
                                                           NodeMeta* meta, const uint64_t* pslot,
                                                           const uint64_t* poff,
                                                           const uint64_t* bins,
                                                           uint64_t* counters) {
  const int64_t u = seg_wave_index();
  if (u >= n) return;
  const int lane = lane_id();
  const uint32_t m = (uint32_t)(k / kSeg);
  uint64_t cnt = pslot[u] & kSlotCountMask;
  const uint64_t beg = poff[u], cap = poff[u + 1] - beg;
  uint64_t lo = G[u * k + lane];
  uint64_t hi = lane + kWave < k ? G[u * k + kWave + lane] : kKeyMax;
  if (cnt == 0) return;
  uint64_t* cs = counters + (u & (kStripes - 1)) * C_SLOTS;
  if (cnt > cap) {  // cannot happen: a segment of the proposal array holds what its node can receive
    if (lane == 0)
      atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_OVERFLOW), (unsigned long long)(cnt - cap));
    cnt = cap;
  }
  // the merged row splits into its segments: a stable compaction per class keeps the order
  uint64_t seg[kMaxSegments];
#pragma unroll
  for (uint32_t r = 0; r < (uint32_t)kMaxSegments; ++r) {
    seg[r] = kKeyMax;
    if (r < m) {  // uniform
      const bool keep_lo = entry_id(lo) % m == r;
      const bool keep_hi = hi != kKeyMax && entry_id(hi) % m == r;
      const int c0 = __popcll(__ballot(keep_lo));
      const uint64_t a = wave_compact(lo, keep_lo, kKeyMax, lane);
      const uint64_t b = wave_compact(hi, keep_hi, kKeyMax, lane);
      const int from = lane - c0;
      const uint64_t b_shift = __shfl(b, from < 0 ? 0 : from, kWave);
      seg[r] = lane < c0 ? a : (lane < kSeg ? b_shift : kKeyMax);
    }
  }
  bool changed = false;
  for (uint64_t c = 0; c < cnt; c += kWave) {
    const uint64_t pk = (c + lane < cnt) ? bins[beg + c + lane] : kKeyMax;
#pragma unroll
    for (uint32_t r = 0; r < (uint32_t)kMaxSegments; ++r) {
      if (r < m) {  // uniform
        uint64_t mine = (pk != kKeyMax && entry_id(pk) % m == r) ? pk : kKeyMax;
        bool any;
        mine = filter_candidates(mine, seg[r], kSeg, lane, any);
        if (any) {
          seg[r] = wave_merge_smallest(seg[r], mine, lane);
          if (lane >= kSeg) seg[r] = kKeyMax;
          changed = true;
        }
      }
    }
  }
  if (!changed) return;
  // "as the iteration is completed, all the segments ... will be merged into one"
  const uint64_t s1 = __shfl(seg[1], lane & (kSeg - 1), kWave);
  const uint64_t s3 = __shfl(seg[3], lane & (kSeg - 1), kWave);
  lo = lane < kSeg ? seg[0] : s1;
  hi = lane < kSeg ? seg[2] : s3;
  sort128(lo, hi, lane);
  const uint64_t adm0 = __ballot((lo & 2ull) != 0);
  const uint64_t adm1 = __ballot(lane + kWave < k && (hi & 2ull) != 0);
  G[u * k + lane] = lo & ~2ull;
  if (lane + kWave < k) G[u * k + kWave + lane] = hi & ~2ull;
  const int last = k - 1;
  if (lane == (last & 63)) meta[u].kth = entry_code(last < kWave ? lo : hi);
  if (lane == 0)
    atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_INSERTS),
              (unsigned long long)(__popcll(adm0) + __popcll(adm1)));
}

}  // namespace

hipError_t launch_init_random_segmented(const Shape& sh, const DevState& ds, uint64_t seed,
                                        hipStream_t st) {
  const dim3 grid = seg_blocks(sh.n);
  const uint64_t base = hash_base(seed, kTagInit);
  const VecSrc vs{sh.vec_a, sh.vec_b, sh.split, sh.d, sh.norms};
  switch (sh.metric) {
    case kL2F32:
      k_init_random_segmented<kL2F32><<<grid, kSGB, 0, st>>>(vs, sh.n, sh.k, base, ds.G, ds.meta);
      break;
    case kAngularF32:
      k_init_random_segmented<kAngularF32><<<grid, kSGB, 0, st>>>(vs, sh.n, sh.k, base, ds.G,
                                                                  ds.meta);
      break;
    case kChi2F32:
      k_init_random_segmented<kChi2F32><<<grid, kSGB, 0, st>>>(vs, sh.n, sh.k, base, ds.G, ds.meta);
      break;
    case kCosineF32:
      k_init_random_segmented<kCosineF32><<<grid, kSGB, 0, st>>>(vs, sh.n, sh.k, base, ds.G,
                                                                 ds.meta);
      break;
    default:
      k_init_random_segmented<kL2U8><<<grid, kSGB, 0, st>>>(vs, sh.n, sh.k, base, ds.G, ds.meta);
  }
  return hipGetLastError();
}

hipError_t launch_update_segmented(const Shape& sh, const DevState& ds, hipStream_t st) {
  k_update_segmented<<<seg_blocks(sh.n), kSGB, 0, st>>>(sh.n, sh.k, ds.G, ds.meta, ds.pslot,
                                                        ds.poff, ds.bins, ds.counters);
  return hipGetLastError();
}

}  // namespace gnnd
