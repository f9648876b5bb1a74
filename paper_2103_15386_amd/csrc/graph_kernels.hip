// Graph-side kernels of GNND for gfx950: random initial lists, sampling with
// reverse neighbours, the list update, and the copy-in / copy-out helpers.
// One 64-lane wavefront owns one list: a list entry, a sample or a proposal
// lives in one lane, and sorting / merging / compaction are lane networks.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

__device__ inline int64_t wave_global_index() {
  return block_linear() * kWavesPerBlock + wave_id();
}
static inline dim3 blocks_for_waves(int64_t waves) {
  return grid_blocks((waves + kWavesPerBlock - 1) / kWavesPerBlock);
}

__device__ inline void counter_add(uint64_t* counters, int which, int64_t stripe_hint,
                                   uint64_t v) {
  atomicAdd(reinterpret_cast<unsigned long long*>(
                counters + (stripe_hint & (kStripes - 1)) * C_SLOTS + which),
            (unsigned long long)v);
}

// ---------------------------------------------------------------------------
// Alg. 1, first loop: k distinct random neighbours per node, distances, sorted
// ascending by (distance, id), flagged NEW.
template <int METRIC>
__global__ __launch_bounds__(kBlock) void k_init_random(VecSrc vs, int64_t n, int k,
                                                        uint64_t base_hash, uint64_t* G,
                                                        NodeMeta* meta) {
  __shared__ uint32_t tile[kWavesPerBlock][kEvalTileWords];
  const int64_t s = wave_global_index();
  if (s >= n) return;
  const int lane = lane_id();
  uint32_t id = draw_distinct(base_hash, (uint32_t)s, k, (uint32_t)n, 0u, (uint32_t)s, lane);
  const uint32_t code =
      wave_distances<METRIC>(vs, (uint32_t)s, id, lane < k, tile[wave_id()], lane);
  uint64_t e = lane < k ? make_entry(code, id, 1u) : kKeyMax;
  e = wave_sort(e, lane);
  if (lane < k) G[s * k + lane] = e;
  if (lane == k - 1) meta[s].kth = entry_code(e);
}

// ---------------------------------------------------------------------------
// What the reverse candidates of v are ranked by: hash(seed, kind, v, s, iter), ties by s.
__device__ inline uint64_t select_key(uint64_t base, int64_t v, uint32_t s, uint32_t iter) {
  return ((hash3(base, (uint32_t)v, s, iter) >> 32) << 32) | (uint64_t)s;
}

// Sec. 4.1, reverse part and duplicate removal for one list.  `fwd_raw` is the
// list row as loaded (its first nf entries are the forward samples), `first` the
// first 64 reverse candidates (lane < deg).  Of the candidates the 2p - nf with
// the smallest hash(seed, kind, v, s, iter) (ties by s) are appended - the
// paper's "append until the list is full" with the winners chosen by a hash
// instead of by thread timing.  The list is then sorted by id, duplicates are
// dropped and it is written back with -1 behind its end.  Returns its size.
__device__ __forceinline__ int select_list(int64_t v, int p, uint64_t base, uint32_t iter, int32_t* list,
                                  uint32_t fwd_raw, int nf, const int32_t* csr, uint64_t beg,
                                  uint32_t deg, uint32_t first, int lane) {
  const uint32_t fwd = lane < nf ? fwd_raw : kIdMax;
  const int room = 2 * p - nf;
  uint32_t rev = kIdMax;
  int m;
  if (deg <= (uint32_t)room) {
    m = (int)deg;
    if (lane < m) rev = first;
  } else {
    m = room;
    uint64_t best = lane < deg ? select_key(base, v, first, iter) : kKeyMax;
    if (room == kWave / 2 && deg <= (uint32_t)kWave) {
      // The usual case (a full forward part, up to 64 candidates).  Which 32 candidates win
      // is all that matters - the list is sorted by id below - so the network stops where
      // the lower half of the lanes holds the 32 smallest keys: halves sorted up and down
      // (15 stages), then one exchange across the halves, instead of 21 stages.
      best = wave_sort_first<kWave / 2>(best, lane);
      best = vmin(best, xor_lanes(best, kWave / 2, lane));
    } else {
      best = wave_sort(best, lane);
      for (uint32_t c = kWave; c < deg; c += kWave) {
        uint64_t key =
            c + lane < deg ? select_key(base, v, (uint32_t)csr[beg + c + lane], iter) : kKeyMax;
        key = wave_sort(key, lane);
        best = wave_merge_smallest(best, key, lane);
      }
    }
    if (lane < room) rev = (uint32_t)best;
  }
  const int src = lane - nf;
  const uint32_t r = __shfl(rev, src < 0 ? 0 : src, kWave);
  uint32_t val = lane < nf ? fwd : (src < m ? r : kIdMax);
  val = wave_sort_upto(val, lane, nf + m);
  const uint32_t prev = __shfl_up(val, 1, kWave);
  const bool keep = val != kIdMax && (lane == 0 || val != prev);
  const uint64_t mask = __ballot(keep);
  const int count = __popcll(mask);
  if (keep) list[__popcll(mask & lanes_below(lane))] = (int32_t)val;
  if (lane >= count && lane < 2 * p) list[lane] = -1;
  return count;
}

// One wavefront finishes both sample lists of kNodesPerWave nodes.  The kernel is bound by
// the latency of its two dependent rounds of reads (sizes, offsets and list rows, then the
// candidate segments), not by its arithmetic, and it needs few registers: so a wavefront
// requests everything of the first round for all its nodes at once, then everything of the
// second round, and only then works the lists off one node after the other.
constexpr int kNodesPerWave = 4;
__global__ __launch_bounds__(kBlock) void k_rev_select(int64_t n, int p, uint64_t base_new,
                                                       uint64_t base_old, uint32_t iter,
                                                       int32_t* snew, int32_t* sold,
                                                       int32_t* cnew, int32_t* cold,
                                                       const uint64_t* roff_new,
                                                       const uint64_t* roff_old,
                                                       const int32_t* csr_new,
                                                       const int32_t* csr_old,
                                                       uint32_t* capn, uint32_t* capo,
                                                       uint32_t per_new, uint32_t per_old,
                                                       uint64_t* counters) {
  const int64_t v0 = wave_global_index() * kNodesPerWave;
  if (v0 >= n) return;
  const int lane = lane_id();
  const int L = 2 * p;
  int nfn[kNodesPerWave], nfo[kNodesPerWave];
  uint64_t bn[kNodesPerWave], bo[kNodesPerWave];
  uint32_t dn[kNodesPerWave], dO[kNodesPerWave];  // a node's reverse degree is below 2^32
  uint32_t rown[kNodesPerWave], rowo[kNodesPerWave], firstn[kNodesPerWave], firsto[kNodesPerWave];
#pragma unroll
  for (int i = 0; i < kNodesPerWave; ++i) {
    const int64_t v = v0 + i < n ? v0 + i : n - 1;  // beyond the end: the last node again, unused
    nfn[i] = cnew[v];
    nfo[i] = cold[v];
    bn[i] = roff_new[v];
    dn[i] = (uint32_t)(roff_new[v + 1] - bn[i]);
    bo[i] = roff_old[v];
    dO[i] = (uint32_t)(roff_old[v + 1] - bo[i]);
    rown[i] = lane < p ? (uint32_t)snew[v * L + lane] : kIdMax;  // the forward part
    rowo[i] = lane < p ? (uint32_t)sold[v * L + lane] : kIdMax;
  }
#pragma unroll
  for (int i = 0; i < kNodesPerWave; ++i) {
    firstn[i] = (uint32_t)lane < dn[i] ? (uint32_t)csr_new[bn[i] + lane] : kIdMax;
    firsto[i] = (uint32_t)lane < dO[i] ? (uint32_t)csr_old[bo[i] + lane] : kIdMax;
  }
  uint64_t sum_new = 0, sum_old = 0;
#pragma unroll
  for (int i = 0; i < kNodesPerWave; ++i) {
    const int64_t v = v0 + i;
    if (v < n) {  // uniform
      const int cn = select_list(v, p, base_new, iter, snew + v * L, rown[i], nfn[i], csr_new,
                                 bn[i], dn[i], firstn[i], lane);
      const int co = select_list(v, p, base_old, iter, sold + v * L, rowo[i], nfo[i], csr_old,
                                 bo[i], dO[i], firsto[i], lane);
      sum_new += (uint64_t)cn;
      sum_old += (uint64_t)co;
      if (lane == 0) {
        cnew[v] = cn;
        cold[v] = co;
        // v can only sit in the sample list of a node that holds v as a forward
        // sample (deg of them) or that v holds as one (nf): that bounds the number
        // of joins v takes part in, hence the nearest-object results it can
        // receive - two per join as a NEW sample, one as an OLD sample (per_new, per_old;
        // when every pair is proposed: one per possible partner).
        capn[v] = (uint32_t)(per_new * (dn[i] + (uint64_t)nfn[i]));
        capo[v] = (uint32_t)(per_old * (dO[i] + (uint64_t)nfo[i]));
      }
    }
  }
  if (lane == 0) {
    counter_add(counters, C_SUMNEW, v0, sum_new);
    counter_add(counters, C_SUMOLD, v0, sum_old);
  }
}

// ---------------------------------------------------------------------------
// Sec. 4.3 list insertion for all proposals of one destination at once: the
// list becomes the best k, by (distance, id), of its entries and the proposed
// objects, one entry per id - what inserting them one by one under a lock
// gives in any order.  Admitted entries are flagged NEW.
__global__ __launch_bounds__(kBlock) void k_update(int64_t n, int k, uint64_t* G, NodeMeta* meta,
                                                   const uint64_t* pslot, const uint64_t* poff,
                                                   const uint64_t* bins, uint64_t* counters) {
  const int64_t u = wave_global_index();
  if (u >= n) return;
  const int lane = lane_id();
  // everything that needs no other load is requested together (the row too, even
  // if the node turns out to have received nothing): one round trip less
  uint64_t cnt = pslot[u] & kSlotCountMask;
  const uint64_t beg = poff[u], cap = poff[u + 1] - beg;
  uint64_t row = lane < k ? G[u * k + lane] : kKeyMax;
  if (cnt == 0) return;
  if (cnt > cap) {  // cannot happen: a segment is sized by the bound of what its node can receive
    if (lane == 0) counter_add(counters, C_OVERFLOW, u, cnt - cap);
    cnt = cap;
  }
  bool changed = false;
  for (uint64_t c = 0; c < cnt; c += kWave) {
    uint64_t pk = (c + lane < cnt) ? bins[beg + c + lane] : kKeyMax;
    bool any;
    pk = filter_candidates(pk, row, k, lane, any);
    if (!any) continue;
    row = wave_merge_smallest(row, pk, lane);
    if (lane >= k) row = kKeyMax;
    changed = true;
  }
  if (!changed) return;
  const uint64_t admitted = __ballot(lane < k && (row & 2ull));
  if (lane < k) G[u * k + lane] = row & ~2ull;
  if (lane == k - 1) meta[u].kth = entry_code(row);
  if (lane == 0) counter_add(counters, C_INSERTS, u, (uint64_t)__popcll(admitted));
}

// ---------------------------------------------------------------------------
// The same for lists of up to 32 entries, two destinations per wavefront: the lower and the
// upper 32 lanes each own a destination, and every step above runs on 32 lanes - both halves
// by the same instructions, with shorter sorting and merging networks.
__device__ inline uint64_t half_lanes(int lane) {
  return (lane & 32) ? 0xffffffff00000000ull : 0x00000000ffffffffull;
}
// stable compaction inside each half (see wave_compact)
__device__ inline uint64_t half_compact(uint64_t v, bool keep, uint64_t fill, int lane) {
  const uint64_t mask = __ballot(keep) & half_lanes(lane);
  const int nkeep = __popcll(mask);
  const int before = __popcll(mask & lanes_below(lane));
  const int dst = (lane & 32) | (keep ? before : nkeep + ((lane & 31) - before));
  const uint64_t x = keep ? v : fill;
  const uint32_t lo = __builtin_amdgcn_ds_permute(dst << 2, (int)(uint32_t)x);
  const uint32_t hi = __builtin_amdgcn_ds_permute(dst << 2, (int)(uint32_t)(x >> 32));
  return ((uint64_t)hi << 32) | lo;
}
// the 32 smallest of two ascending 32-lane sequences, ascending, in each half
__device__ inline uint64_t half_merge_smallest(uint64_t a_sorted, uint64_t b_sorted, int lane) {
  // value of lane 31 - (lane % 32) of the half: mirror inside the row of 16, then swap the rows
  const uint32_t mlo = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)b_sorted, 0x140, 0xF, 0xF, true);
  const uint32_t mhi =
      (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)(b_sorted >> 32), 0x140, 0xF, 0xF, true);
  const uint64_t br = xor_lanes(((uint64_t)mhi << 32) | mlo, 16, lane);
  uint64_t v = vmin(a_sorted, br);
#pragma unroll
  for (int j = 16; j > 0; j >>= 1) {
    const uint64_t o = xor_lanes(v, j, lane);
    v = exchange(v, o, (lane & j) == 0);
  }
  return v;
}
// filter_candidates on 32 lanes, in two parts; `row` holds k <= 32 ascending entries per half.
// First part: what is not closer than the list's last entry or already in the list becomes
// kKeyMax (where it stands).
__device__ inline uint64_t half_drop_known(uint64_t pk, uint64_t row, int k, int lane) {
  const int base = lane & 32;
  const uint64_t last = __shfl(row, base | (k - 1), kWave);
  if (pk != kKeyMax && entry_key(pk) >= entry_key(last)) pk = kKeyMax;
  if (__ballot(pk != kKeyMax) == 0ull) return pk;
  const uint64_t kk = entry_key(pk);
  int pos = 0;
#pragma unroll
  for (int step = 16; step > 0; step >>= 1) {
    const uint64_t r = __shfl(row, base | (pos + step - 1), kWave);
    pos += (entry_key(r) < kk) ? step : 0;
  }
  if (entry_key(__shfl(row, base | pos, kWave)) == kk) pk = kKeyMax;
  return pk;
}
// Second part: the survivors, already at the front of their half (`count` = the larger
// number of them in the two halves), ascending and without repeats.
__device__ inline uint64_t half_sort_unique(uint64_t pk, int count, int lane) {
  const int l32 = lane & 31;
  // the networks over up to 32 lanes never cross the halves; the in-half lane number makes
  // both halves ascend
  if (count > 16) pk = wave_sort_first<32>(pk, l32);
  else if (count > 8) pk = wave_sort_first<16>(pk, l32);
  else if (count > 4) pk = wave_sort_first<8>(pk, l32);
  else if (count > 2) pk = wave_sort_first<4>(pk, l32);
  else if (count > 1) pk = wave_sort_first<2>(pk, l32);
  const uint64_t prev = __shfl_up(pk, 1, kWave);
  const bool rep = l32 > 0 && pk != kKeyMax && entry_key(pk) == entry_key(prev);
  if (__ballot(rep) != 0ull) pk = half_compact(pk, !rep, kKeyMax, lane);
  return pk;
}

// The work on one pair of destinations (one per half): `row`, `cnt`, `beg` as loaded, `pa` /
// `pb` the first 64 proposals of each destination (two per lane, kKeyMax beyond cnt).
__device__ inline void update_pair(int64_t u, bool live, int k, uint64_t cnt, uint64_t beg,
                                   uint64_t row, uint64_t pa, uint64_t pb, uint64_t* G,
                                   NodeMeta* meta, const uint64_t* bins, uint64_t* counters,
                                   int lane) {
  const int l32 = lane & 31;
  if (__ballot(cnt != 0) == 0ull) return;
  const uint64_t cnt_other = __shfl(cnt, lane ^ 32, kWave);
  const uint64_t rounds = cnt > cnt_other ? cnt : cnt_other;
  const uint64_t mine_mask = half_lanes(lane);
  bool changed = false;
  // survivors (at the front of their half, `count` at most in either half) into the row
  auto admit = [&](uint64_t pk, int count) {
    pk = half_sort_unique(pk, count, lane);
    const bool mine = (__ballot(pk != kKeyMax) & mine_mask) != 0ull;
    row = half_merge_smallest(row, pk, lane);  // a half without survivors keeps its row
    if (l32 >= k) row = kKeyMax;
    changed = changed || mine;
  };
  // A round takes 64 proposals per destination, two per lane.  Few of them survive the cheap
  // tests as a rule: when the survivors of both registers fit one half they go through one
  // sorting and one merging network, otherwise the second register waits for the first.
  for (uint64_t c = 0; c < rounds; c += 64) {
    if (c > 0) {
      pa = (c + l32 < cnt) ? bins[beg + c + l32] : kKeyMax;
      pb = (c + 32 + l32 < cnt) ? bins[beg + c + 32 + l32] : kKeyMax;
    }
    pa = half_drop_known(pa, row, k, lane);
    pb = half_drop_known(pb, row, k, lane);
    const uint64_t left_a = __ballot(pa != kKeyMax), left_b = __ballot(pb != kKeyMax);
    if ((left_a | left_b) == 0ull) continue;
    const int na = __popcll(left_a & mine_mask), nb = __popcll(left_b & mine_mask);
    const int na_max = vmax(__popcll(left_a & 0xffffffffull), __popcll(left_a >> 32));
    pa = half_compact(pa, pa != kKeyMax, kKeyMax, lane);
    if (left_b == 0ull) {
      admit(pa, na_max);
    } else if (__ballot(na + nb > 32) == 0ull) {
      pb = half_compact(pb, pb != kKeyMax, kKeyMax, lane);
      const int src = l32 - na;
      const uint64_t shifted = __shfl(pb, (lane & 32) | (src < 0 ? 0 : src), kWave);
      const int n0 = __popcll(left_a & 0xffffffffull) + __popcll(left_b & 0xffffffffull);
      const int n1 = __popcll(left_a >> 32) + __popcll(left_b >> 32);
      admit(l32 < na ? pa : shifted, vmax(n0, n1));
    } else {
      if (left_a != 0ull) admit(pa, na_max);
      // the list has changed: the second register takes the cheap tests again
      pb = half_drop_known(pb, row, k, lane);
      const uint64_t left = __ballot(pb != kKeyMax);
      if (left != 0ull) {
        pb = half_compact(pb, pb != kKeyMax, kKeyMax, lane);
        admit(pb, vmax(__popcll(left & 0xffffffffull), __popcll(left >> 32)));
      }
    }
  }
  const uint64_t admitted = __ballot(l32 < k && (row & 2ull)) & mine_mask;
  if (changed && live) {
    if (l32 < k) G[u * k + l32] = row & ~2ull;
    if (l32 == k - 1) meta[u].kth = entry_code(row);
    if (l32 == 0) counter_add(counters, C_INSERTS, u, (uint64_t)__popcll(admitted));
  }
}

// One pair of destinations per wavefront.  (Unlike k_rev_select this kernel is bound by
// vector-instruction issue: with two pairs per wavefront and both rounds of reads requested up
// front it was slower, 3.4 against 3.1 ms per build on the benchmark workload.)
constexpr int kPairsPerWave = 1;
__global__ __launch_bounds__(kBlock) void k_update_pairs(int64_t n, int k, uint64_t* G,
                                                         NodeMeta* meta, const uint64_t* pslot,
                                                         const uint64_t* poff,
                                                         const uint64_t* bins, uint64_t* counters) {
  const int lane = lane_id(), l32 = lane & 31;
  const int64_t u0 = wave_global_index() * (2 * kPairsPerWave) + (lane >> 5);
  if (u0 - (lane >> 5) >= n) return;  // the whole wavefront lies beyond the last node
  int64_t u[kPairsPerWave];
  bool live[kPairsPerWave];
  uint64_t cnt[kPairsPerWave], beg[kPairsPerWave], row[kPairsPerWave];
  uint64_t pa[kPairsPerWave], pb[kPairsPerWave];
#pragma unroll
  for (int j = 0; j < kPairsPerWave; ++j) {
    u[j] = u0 + 2 * j;
    live[j] = u[j] < n;
    cnt[j] = live[j] ? pslot[u[j]] & kSlotCountMask : 0;
    beg[j] = live[j] ? poff[u[j]] : 0;
    const uint64_t cap = live[j] ? poff[u[j] + 1] - beg[j] : 0;
    row[j] = (live[j] && l32 < k) ? G[u[j] * k + l32] : kKeyMax;
    if (cnt[j] > cap) {  // cannot happen: a segment is sized by the bound of what its node can receive
      if (l32 == 0) counter_add(counters, C_OVERFLOW, u[j], cnt[j] - cap);
      cnt[j] = cap;
    }
  }
#pragma unroll
  for (int j = 0; j < kPairsPerWave; ++j) {
    pa[j] = (l32 < cnt[j]) ? bins[beg[j] + l32] : kKeyMax;
    pb[j] = (32 + l32 < cnt[j]) ? bins[beg[j] + 32 + l32] : kKeyMax;
  }
#pragma unroll
  for (int j = 0; j < kPairsPerWave; ++j)
    update_pair(u[j], live[j], k, cnt[j], beg[j], row[j], pa[j], pb[j], G, meta, bins, counters,
                lane);
}

// ---------------------------------------------------------------------------
template <bool FLOAT>
__global__ __launch_bounds__(kBlock) void k_get_graph(int64_t total, const uint64_t* G,
                                                      int32_t* ids, void* dist, uint8_t* isnew,
                                                      int32_t id_offset) {
  const int64_t i = block_linear() * kBlock + threadIdx.x;
  if (i >= total) return;
  const uint64_t e = G[i];
  if (ids) ids[i] = (int32_t)entry_id(e) + id_offset;
  if (isnew) isnew[i] = (uint8_t)(e & 1ull);
  if (dist) {
    if (FLOAT) reinterpret_cast<float*>(dist)[i] = unord_f32(entry_code(e));
    else reinterpret_cast<int32_t*>(dist)[i] = unord_i32(entry_code(e));
  }
}

// An id that is no node of the graph, or the row's own node, would later be
// used as a row number: it raises `bad` and is replaced by a valid id, so that
// nothing can read out of bounds even if the caller ignores the error.
template <bool FLOAT>
__global__ __launch_bounds__(kBlock) void k_set_graph(int64_t total, int64_t n, int k, uint64_t* G,
                                                      NodeMeta* meta, const int32_t* ids,
                                                      const void* dist, const uint8_t* isnew,
                                                      int* bad) {
  const int64_t i = block_linear() * kBlock + threadIdx.x;
  if (i >= total) return;
  uint32_t code = FLOAT ? ord_f32(reinterpret_cast<const float*>(dist)[i])
                        : ord_i32(reinterpret_cast<const int32_t*>(dist)[i]);
  const int64_t row = i / k;
  uint32_t id = (uint32_t)ids[i];
  if ((int64_t)id >= n || (int64_t)id == row) {
    atomicOr(bad, 1);
    id = (uint32_t)((row + 1 + i % k) % n);
  }
  G[i] = make_entry(code, id, isnew ? (uint32_t)(isnew[i] & 1) : 0u);
  if ((i % k) == k - 1) meta[i / k].kth = code;
}

// Copy the proposal segments out: slot j of destination u's segment holds u and
// the proposed (object, distance) when filled, -1 otherwise.
template <bool FLOAT>
__global__ __launch_bounds__(kBlock) void k_get_proposals(int64_t n, const uint64_t* pslot,
                                                          const uint64_t* poff,
                                                          const uint64_t* bins, int32_t* u_out,
                                                          int32_t* v_out, void* dist) {
  const int64_t u = wave_global_index();
  if (u >= n) return;
  const uint64_t beg = poff[u], cap = poff[u + 1] - beg, cnt = pslot[u] & kSlotCountMask;
  for (uint64_t i = lane_id(); i < cap; i += kWave) {
    const bool have = i < cnt;
    const uint64_t e = have ? bins[beg + i] : 0ull;
    u_out[beg + i] = have ? (int32_t)u : -1;
    v_out[beg + i] = have ? (int32_t)entry_id(e) : -1;
    if (FLOAT) reinterpret_cast<float*>(dist)[beg + i] = have ? unord_f32(entry_code(e)) : 0.f;
    else reinterpret_cast<int32_t*>(dist)[beg + i] = have ? unord_i32(entry_code(e)) : 0;
  }
}

// Slots beyond the last segment (the segments need not fill the whole array).
__global__ __launch_bounds__(kBlock) void k_fill_i32(int32_t* p, const uint64_t* from,
                                                     int64_t end, int32_t value) {
  const int64_t i = (int64_t)(*from) + block_linear() * kBlock + threadIdx.x;
  if (i < end) p[i] = value;
}

__global__ __launch_bounds__(kBlock) void k_zero_u32(uint32_t* p, size_t count) {
  const size_t i = (size_t)block_linear() * kBlock + threadIdx.x;
  if (i < count) p[i] = 0u;
}

__global__ __launch_bounds__(kBlock) void k_copy_u64(uint64_t* dst, const uint64_t* src,
                                                     size_t count) {
  const size_t i = (size_t)block_linear() * kBlock + threadIdx.x;
  if (i < count) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// GGM, Alg. 3 "Divide" + "Append": keep the first ceil(k/2) entries (OLD), set
// the rest aside, refill with floor(k/2) random objects of the other set (NEW)
// and restore the (distance, id) order.
template <int METRIC>
__global__ __launch_bounds__(kBlock) void k_merge_init(VecSrc vs, int64_t n, MergeIds mi, int k,
                                                       uint64_t base_hash, const int32_t* ids1,
                                                       const void* dist1, const int32_t* ids2,
                                                       const void* dist2, uint64_t* G,
                                                       NodeMeta* meta, uint64_t* aside) {
  __shared__ uint32_t tile[kWavesPerBlock][kEvalTileWords];
  const int64_t s = wave_global_index();
  if (s >= n) return;
  const int lane = lane_id();
  const int64_t n1 = mi.n1;
  const bool first = s < n1;
  const int64_t loc = first ? s : s - n1;
  const int32_t* sid = (first ? ids1 : ids2) + loc * k;
  const void* sdist = first ? dist1 : dist2;
  const int keep = (k + 1) / 2, fill = k / 2;
  uint32_t id_in = 0, code_in = 0;
  if (lane < k) {
    id_in = mi.to_internal(sid[lane]);  // collection id -> numbering of this merge
    code_in = METRIC == kL2U8
                  ? ord_i32(reinterpret_cast<const int32_t*>(sdist)[loc * k + lane])
                  : ord_f32(reinterpret_cast<const float*>(sdist)[loc * k + lane]);
  }
  if (lane >= keep && lane < k) aside[s * fill + (lane - keep)] = make_entry(code_in, id_in, 0u);
  const uint32_t draw = draw_distinct(base_hash, (uint32_t)s, fill,
                                      (uint32_t)(first ? n - n1 : n1), first ? (uint32_t)n1 : 0u,
                                      0xffffffffu, lane);
  const int src = lane - keep;
  const uint32_t did = __shfl(draw, src < 0 ? 0 : src, kWave);
  const uint32_t code = wave_distances<METRIC>(vs, (uint32_t)s, did, lane >= keep && lane < k,
                                               tile[wave_id()], lane);
  uint64_t e = kKeyMax;
  if (lane < keep) e = make_entry(code_in, id_in, 0u);
  else if (lane < k) e = make_entry(code, did, 1u);
  e = wave_sort(e, lane);
  if (lane < k) G[s * k + lane] = e;
  if (lane == k - 1) meta[s].kth = entry_code(e);
}

// GGM, Alg. 3 "Merge and Sort": best k of the refined list and the set-aside
// half, handed out under collection ids, ascending by (distance, collection id).
template <bool FLOAT>
__global__ __launch_bounds__(kBlock) void k_merge_final(int64_t n, MergeIds mi, int k,
                                                        const uint64_t* G, const uint64_t* aside,
                                                        int32_t* ids_out, void* dist_out) {
  const int64_t s = wave_global_index();
  if (s >= n) return;
  const int lane = lane_id();
  const int fill = k / 2;
  uint64_t row = lane < k ? G[s * k + lane] : kKeyMax;
  uint64_t pk = lane < fill ? aside[s * fill + lane] : kKeyMax;
  // the set-aside entries may tie with the list's last entry: compare on the
  // full (distance, id) key, which filter_candidates does
  bool any;
  pk = filter_candidates(pk, row, k, lane, any);
  if (any) {
    row = wave_merge_smallest(row, pk, lane);
  }
  // renumber, then restore the order under the new ids (only ties can move)
  row = lane < k ? make_entry(entry_code(row), (uint32_t)mi.to_global(entry_id(row)), 0u)
                 : kKeyMax;
  row = wave_sort(row, lane);
  if (lane < k) {
    ids_out[s * k + lane] = (int32_t)entry_id(row);
    if (FLOAT) reinterpret_cast<float*>(dist_out)[s * k + lane] = unord_f32(entry_code(row));
    else reinterpret_cast<int32_t*>(dist_out)[s * k + lane] = unord_i32(entry_code(row));
  }
}

// ---------------------------------------------------------------------------
// Exhaustive exact K-NN of a query node (ground truth for Recall@K): each wave
// scans a quarter of the data set, one candidate per lane, and keeps the best
// 64 in its lanes; the four lists are merged at the end.
template <int METRIC>
__global__ __launch_bounds__(kBlock) void k_exact_knn(const void* vec, int64_t n, int d,
                                                      const int32_t* queries, int K,
                                                      int32_t* ids_out, void* dist_out) {
  using D = DistOf<METRIC>;
  using T = typename D::elem;
  __shared__ uint64_t part[kWavesPerBlock][kWave];
  const int lane = lane_id();
  const int wave = wave_id();
  const int64_t q = blockIdx.x;
  const uint32_t s = (uint32_t)queries[q];
  const T* base = reinterpret_cast<const T*>(vec);
  // a query id that is no node reads nothing and gets the "none" answer (-1, largest distance)
  const bool valid = (int64_t)s < n;
  const T* qrow = base + (valid ? (int64_t)s * d : 0);
  uint64_t best = kKeyMax;  // ascending in lanes; lanes >= K stay unused
  for (int64_t c0 = (int64_t)wave * kWave; valid && c0 < n; c0 += kBlock) {
    const int64_t c = c0 + lane;
    uint64_t key = kKeyMax;
    if (c < n && c != (int64_t)s) {
      uint32_t code = D::eval(qrow, base + c * d, d);
      key = ((uint64_t)code << 32) | (uint64_t)c;
    }
    const uint64_t last = readlane64(best, K - 1);
    if (key >= last) key = kKeyMax;
    if (__ballot(key != kKeyMax) == 0ull) continue;
    key = wave_sort(key, lane);
    best = wave_merge_smallest(best, key, lane);
    if (lane >= K) best = kKeyMax;
  }
  part[wave][lane] = best;
  __syncthreads();
  if (wave == 0) {
    for (int w = 1; w < kWavesPerBlock; ++w) {
      best = wave_merge_smallest(best, part[w][lane], lane);
      if (lane >= K) best = kKeyMax;
    }
    if (lane < K) {
      const bool have = best != kKeyMax;
      ids_out[q * K + lane] = have ? (int32_t)(uint32_t)best : -1;
      uint32_t code = (uint32_t)(best >> 32);
      if (METRIC == kL2U8)
        reinterpret_cast<int32_t*>(dist_out)[q * K + lane] = have ? unord_i32(code) : 0x7fffffff;
      else
        reinterpret_cast<float*>(dist_out)[q * K + lane] =
            have ? unord_f32(code) : __uint_as_float(0x7f800000u);
    }
  }
}

// ---------------------------------------------------------------------------
// Exclusive scan, three passes: per-block scan of 1024 elements, scan of the
// block sums by one block, add-back.
constexpr int kScanPerThread = 4;
constexpr int kScanPerBlock = kBlock * kScanPerThread;

__device__ inline uint64_t block_exclusive_scan(uint64_t v, uint64_t* total) {
  __shared__ uint64_t wsum[kWavesPerBlock];
  const int lane = lane_id();
  const int wave = wave_id();
  uint64_t inc = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    uint64_t o = __shfl_up(inc, off, kWave);
    if (lane >= off) inc += o;
  }
  if (lane == kWave - 1) wsum[wave] = inc;
  __syncthreads();
  uint64_t before = 0, all = 0;
  for (int w = 0; w < kWavesPerBlock; ++w) {
    if (w < wave) before += wsum[w];
    all += wsum[w];
  }
  __syncthreads();
  *total = all;
  return before + inc - v;
}

__global__ __launch_bounds__(kBlock) void k_scan_local(const uint32_t* in, const uint32_t* in2,
                                                       uint64_t* out, uint64_t* bsum,
                                                       uint64_t* counters, int64_t count) {
  const int64_t i0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kScanPerThread;
  uint32_t v[kScanPerThread];
  uint64_t sum = 0;
#pragma unroll
  for (int j = 0; j < kScanPerThread; ++j) {
    v[j] = (i0 + j < count) ? in[i0 + j] + (in2 ? in2[i0 + j] : 0u) : 0u;
    sum += v[j];
    // a segment longer than the count field of the slot word can hold is reported
    if (counters && v[j] > kSlotCountMask) counter_add(counters, C_OVERFLOW, i0 + j, v[j]);
  }
  uint64_t total;
  uint64_t run = block_exclusive_scan(sum, &total);
#pragma unroll
  for (int j = 0; j < kScanPerThread; ++j) {
    if (i0 + j <= count) out[i0 + j] = run;
    run += v[j];
  }
  if (threadIdx.x == 0) bsum[blockIdx.x] = total;
}

__global__ __launch_bounds__(kBlock) void k_scan_bsum(uint64_t* bsum, int64_t nb) {
  uint64_t carry = 0;
  for (int64_t c = 0; c < nb; c += kBlock) {
    const int64_t i = c + threadIdx.x;
    uint64_t v = i < nb ? bsum[i] : 0;
    uint64_t total;
    uint64_t ex = block_exclusive_scan(v, &total);
    if (i < nb) bsum[i] = carry + ex;
    carry += total;
  }
}

__global__ __launch_bounds__(kBlock) void k_scan_add(uint64_t* out, uint64_t* packed,
                                                     const uint64_t* bsum, int64_t count) {
  const int64_t i0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * kScanPerThread;
  const uint64_t add = bsum[blockIdx.x];
#pragma unroll
  for (int j = 0; j < kScanPerThread; ++j)
    if (i0 + j <= count) {
      const uint64_t v = out[i0 + j] + add;
      out[i0 + j] = v;
      // slot word of element i0 + j: its offset, nothing received yet
      if (packed && i0 + j < count) packed[i0 + j] = v << kSlotCountBits;
    }
}

size_t scan_tmp_elems(int64_t count) { return (size_t)((count + 1 + kScanPerBlock - 1) / kScanPerBlock); }

hipError_t launch_scan(const uint32_t* in, const uint32_t* in2, uint64_t* out, uint64_t* packed,
                       uint64_t* counters, uint64_t* tmp, int64_t count, hipStream_t st) {
  const int64_t nb = (count + 1 + kScanPerBlock - 1) / kScanPerBlock;
  k_scan_local<<<(unsigned)nb, kBlock, 0, st>>>(in, in2, out, tmp, counters, count);
  k_scan_bsum<<<1, kBlock, 0, st>>>(tmp, nb);
  k_scan_add<<<(unsigned)nb, kBlock, 0, st>>>(out, packed, tmp, count);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
static VecSrc vec_src(const Shape& sh) {
  return VecSrc{sh.vec_a, sh.vec_b, sh.split, sh.d, sh.norms};
}

hipError_t launch_zero_u32(uint32_t* p, size_t count, hipStream_t st) {
  if (count == 0) return hipSuccess;
  k_zero_u32<<<grid_blocks((int64_t)((count + kBlock - 1) / kBlock)), kBlock, 0, st>>>(p, count);
  return hipGetLastError();
}

// A small copy inside the stream of kernels (the runtime's own copy leaves the GPU idle for
// some 10 microseconds around it).
hipError_t launch_copy_u64(uint64_t* dst, const uint64_t* src, size_t count, hipStream_t st) {
  if (count == 0) return hipSuccess;
  k_copy_u64<<<grid_blocks((int64_t)((count + kBlock - 1) / kBlock)), kBlock, 0, st>>>(dst, src,
                                                                                      count);
  return hipGetLastError();
}

// Squared norm of every row, one fused multiply-add per dimension in dimension
// order (what the cosine distance divides by).  A wavefront takes 64 rows: chunks
// of kEvalChunk dimensions go through LDS with coalesced reads (8 lanes per row
// chunk), then each lane adds up its own row.
__global__ __launch_bounds__(kBlock) void k_row_norms(VecSrc vs, int64_t n, float* norms) {
  __shared__ float tile[kWavesPerBlock][64 * kEvalStride];
  const int lane = lane_id();
  float* my = tile[wave_id()];
  const int64_t row0 = (block_linear() * kWavesPerBlock + wave_id()) * 64;
  if (row0 >= n) return;
  const int d = vs.d;
  const int part = lane & 7, rsel = lane >> 3;
  float acc = 0.f;
  for (int d0 = 0; d0 < d; d0 += kEvalChunk) {
#pragma unroll
    for (int r0 = 0; r0 < 64; r0 += 8) {
      const int r = r0 + rsel;
      if (row0 + r < n) {
        const float* src = vs.row<float>((uint32_t)(row0 + r));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int j = d0 + part * 4 + q;
          my[r * kEvalStride + part * 4 + q] = j < d ? src[j] : 0.f;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int width = d - d0 < kEvalChunk ? d - d0 : kEvalChunk;
    for (int j = 0; j < width; ++j) {
      const float x = my[lane * kEvalStride + j];
      acc = __fmaf_rn(x, x, acc);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if (row0 + lane < n) norms[row0 + lane] = acc;
}

hipError_t launch_row_norms(const Shape& sh, float* norms, hipStream_t st) {
  const int64_t waves = (sh.n + 63) / 64;
  k_row_norms<<<grid_blocks((waves + kWavesPerBlock - 1) / kWavesPerBlock), kBlock, 0, st>>>(
      vec_src(sh), sh.n, norms);
  return hipGetLastError();
}

hipError_t launch_init_random(const Shape& sh, const DevState& ds, uint64_t seed,
                              hipStream_t st) {
  if (sh.segments > 1) return launch_init_random_segmented(sh, ds, seed, st);
  if (sh.k > kWave) return launch_init_random_wide(sh, ds, seed, st);
  const dim3 grid = blocks_for_waves(sh.n);
  const uint64_t base = hash_base(seed, kTagInit);
  switch (sh.metric) {
    case kL2F32:
      k_init_random<kL2F32><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, sh.k, base, ds.G, ds.meta);
      break;
    case kAngularF32:
      k_init_random<kAngularF32><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, sh.k, base, ds.G,
                                                          ds.meta);
      break;
    case kChi2F32:
      k_init_random<kChi2F32><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, sh.k, base, ds.G,
                                                       ds.meta);
      break;
    case kCosineF32:
      k_init_random<kCosineF32><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, sh.k, base, ds.G,
                                                         ds.meta);
      break;
    default:
      k_init_random<kL2U8><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, sh.k, base, ds.G, ds.meta);
  }
  return hipGetLastError();
}

hipError_t launch_sample(const Shape& sh, const DevState& ds, uint64_t seed, uint32_t iter,
                         hipStream_t st) {
  // forward sampling, and the reverse candidates grouped by target (two-level counting sort)
  hipError_t e = launch_sample_buckets(sh, ds, st);
  if (e != hipSuccess) return e;
  if (2 * sh.p > kWave) {  // two list entries per lane
    e = launch_rev_select_long(sh, ds, seed, iter, st);
    if (e != hipSuccess) return e;
    return launch_scan(ds.capn, ds.capo, ds.poff, ds.pslot, ds.counters, ds.scan_tmp, sh.n, st);
  }
  k_rev_select<<<blocks_for_waves((sh.n + kNodesPerWave - 1) / kNodesPerWave), kBlock, 0, st>>>(
      sh.n, sh.p, hash_base(seed, kTagRevNew), hash_base(seed, kTagRevOld), iter, ds.snew,
      ds.sold, ds.cnew, ds.cold, ds.roff_new, ds.roff_old, ds.csr_new, ds.csr_old, ds.capn,
      ds.capo, (uint32_t)sh.slots_new_per_appearance(), (uint32_t)sh.slots_old_per_appearance(),
      ds.counters);
  // one segment of the proposal array per destination, sized by its bound
  return launch_scan(ds.capn, ds.capo, ds.poff, ds.pslot, ds.counters, ds.scan_tmp, sh.n, st);
}

hipError_t launch_update(const Shape& sh, const DevState& ds, hipStream_t st) {
  if (sh.segments > 1) return launch_update_segmented(sh, ds, st);
  if (sh.k > kWave) return launch_update_wide(sh, ds, st);
  if (sh.k <= 32)
    k_update_pairs<<<blocks_for_waves((sh.n + 2 * kPairsPerWave - 1) / (2 * kPairsPerWave)), kBlock, 0, st>>>(
        sh.n, sh.k, ds.G, ds.meta, ds.pslot, ds.poff, ds.bins, ds.counters);
  else
    k_update<<<blocks_for_waves(sh.n), kBlock, 0, st>>>(sh.n, sh.k, ds.G, ds.meta, ds.pslot,
                                                        ds.poff, ds.bins, ds.counters);
  return hipGetLastError();
}

hipError_t launch_get_graph(const Shape& sh, const DevState& ds, int32_t* ids, void* dist,
                            uint8_t* isnew, int32_t id_offset, hipStream_t st) {
  const int64_t total = sh.n * sh.k;
  const dim3 grid = grid_blocks((total + kBlock - 1) / kBlock);
  if (sh.metric == kL2U8)
    k_get_graph<false><<<grid, kBlock, 0, st>>>(total, ds.G, ids, dist, isnew, id_offset);
  else
    k_get_graph<true><<<grid, kBlock, 0, st>>>(total, ds.G, ids, dist, isnew, id_offset);
  return hipGetLastError();
}

hipError_t launch_set_graph(const Shape& sh, const DevState& ds, const int32_t* ids,
                            const void* dist, const uint8_t* isnew, int* bad_flag_dev,
                            hipStream_t st) {
  const int64_t total = sh.n * sh.k;
  const dim3 grid = grid_blocks((total + kBlock - 1) / kBlock);
  if (sh.metric == kL2U8)
    k_set_graph<false><<<grid, kBlock, 0, st>>>(total, sh.n, sh.k, ds.G, ds.meta, ids, dist, isnew,
                                                bad_flag_dev);
  else
    k_set_graph<true><<<grid, kBlock, 0, st>>>(total, sh.n, sh.k, ds.G, ds.meta, ids, dist, isnew,
                                               bad_flag_dev);
  return hipGetLastError();
}

hipError_t launch_get_proposals(const Shape& sh, const DevState& ds, int32_t* u, int32_t* v,
                                void* dist, hipStream_t st) {
  const dim3 grid = blocks_for_waves(sh.n);
  if (sh.metric == kL2U8)
    k_get_proposals<false><<<grid, kBlock, 0, st>>>(sh.n, ds.pslot, ds.poff, ds.bins, u, v, dist);
  else
    k_get_proposals<true><<<grid, kBlock, 0, st>>>(sh.n, ds.pslot, ds.poff, ds.bins, u, v, dist);
  const int64_t slots = sh.slots();
  const dim3 g2 = grid_blocks((slots + kBlock - 1) / kBlock);
  k_fill_i32<<<g2, kBlock, 0, st>>>(u, ds.poff + sh.n, slots, -1);
  k_fill_i32<<<g2, kBlock, 0, st>>>(v, ds.poff + sh.n, slots, -1);
  return hipGetLastError();
}

hipError_t launch_merge_init(const Shape& sh, const DevState& ds, uint64_t seed,
                             const MergeIds& mi, const int32_t* ids1, const void* dist1,
                             const int32_t* ids2, const void* dist2, hipStream_t st) {
  if (sh.k > kWave) return launch_merge_init_wide(sh, ds, seed, mi, ids1, dist1, ids2, dist2, st);
  const dim3 grid = blocks_for_waves(sh.n);
  const uint64_t base = hash_base(seed, kTagMerge);
  switch (sh.metric) {
    case kL2F32:
      k_merge_init<kL2F32><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, mi, sh.k, base, ids1, dist1,
                                                    ids2, dist2, ds.G, ds.meta, ds.aside);
      break;
    case kAngularF32:
      k_merge_init<kAngularF32><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, mi, sh.k, base, ids1,
                                                         dist1, ids2, dist2, ds.G, ds.meta,
                                                         ds.aside);
      break;
    case kChi2F32:
      k_merge_init<kChi2F32><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, mi, sh.k, base, ids1,
                                                      dist1, ids2, dist2, ds.G, ds.meta, ds.aside);
      break;
    case kCosineF32:
      k_merge_init<kCosineF32><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, mi, sh.k, base, ids1,
                                                        dist1, ids2, dist2, ds.G, ds.meta,
                                                        ds.aside);
      break;
    default:
      k_merge_init<kL2U8><<<grid, kBlock, 0, st>>>(vec_src(sh), sh.n, mi, sh.k, base, ids1, dist1,
                                                   ids2, dist2, ds.G, ds.meta, ds.aside);
  }
  return hipGetLastError();
}

hipError_t launch_merge_final(const Shape& sh, const DevState& ds, const MergeIds& mi,
                              int32_t* ids_out, void* dist_out, hipStream_t st) {
  if (sh.k > kWave) return launch_merge_final_wide(sh, ds, mi, ids_out, dist_out, st);
  const dim3 grid = blocks_for_waves(sh.n);
  if (sh.metric == kL2U8)
    k_merge_final<false><<<grid, kBlock, 0, st>>>(sh.n, mi, sh.k, ds.G, ds.aside, ids_out,
                                                  dist_out);
  else
    k_merge_final<true><<<grid, kBlock, 0, st>>>(sh.n, mi, sh.k, ds.G, ds.aside, ids_out,
                                                 dist_out);
  return hipGetLastError();
}

hipError_t launch_exact_knn(const void* vec, int64_t n, int32_t d, int32_t metric,
                            const int32_t* queries, int64_t nq, int32_t K, int32_t* ids_out,
                            void* dist_out, hipStream_t st) {
  if (nq == 0) return hipSuccess;
  const unsigned grid = (unsigned)nq;
  switch (metric) {
    case kL2F32:
      k_exact_knn<kL2F32><<<grid, kBlock, 0, st>>>(vec, n, d, queries, K, ids_out, dist_out);
      break;
    case kAngularF32:
      k_exact_knn<kAngularF32><<<grid, kBlock, 0, st>>>(vec, n, d, queries, K, ids_out, dist_out);
      break;
    case kChi2F32:
      k_exact_knn<kChi2F32><<<grid, kBlock, 0, st>>>(vec, n, d, queries, K, ids_out, dist_out);
      break;
    case kCosineF32:
      k_exact_knn<kCosineF32><<<grid, kBlock, 0, st>>>(vec, n, d, queries, K, ids_out, dist_out);
      break;
    default:
      k_exact_knn<kL2U8><<<grid, kBlock, 0, st>>>(vec, n, d, queries, K, ids_out, dist_out);
  }
  return hipGetLastError();
}

}  // namespace gnnd
