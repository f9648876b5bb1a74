// Sample lists of 65..128 objects (sample number p of 33..64; the paper varies p
// up to 42, Sec. 6.3).  Two kernels differ from the short-list path:
//  - k_rev_select_long: reverse part, duplicate removal and id order of a sample
//    list (Sec. 4.1) with two list entries per lane, like the long k-NN lists;
//  - k_join_long: cross-matching and nearest-object search (Sec. 4.2, 4.3, Alg. 2)
//    of one node per workgroup, the distance matrix evaluated in blocks of
//    64 x 64 pairs, canonical arithmetic (one fused multiply-add per dimension in
//    dimension order; exact int32 for bytes).
// Forward sampling, the reverse-candidate transpose, the list update and both
// merge steps are the general kernels.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

namespace {

constexpr int kLB = 256;
constexpr int kWavesPerLB = kLB / kWave;

__device__ inline void counter_add_long(uint64_t* counters, int which, int64_t stripe_hint,
                                        uint64_t v) {
  atomicAdd(reinterpret_cast<unsigned long long*>(
                counters + (stripe_hint & (kStripes - 1)) * C_SLOTS + which),
            (unsigned long long)v);
}

// One sample list of up to 128 objects.  `fwd_raw` holds the forward samples (lane <
// nf <= 64); of the `deg` reverse candidates csr[beg..] the 2p - nf with the smallest
// hash(seed, kind, v, s, iter) (ties by s) join them, all of them when they fit.  The
// list is then sorted by id, duplicates are dropped, and it is written back with -1
// behind its end.  Returns its size.
__device__ inline int select_list_long(int64_t v, int p, uint64_t base, uint32_t iter,
                                       int32_t* list, uint32_t fwd_raw, int nf,
                                       const int32_t* csr, uint64_t beg, uint64_t deg, int lane) {
  const int room = 2 * p - nf;  // 1..128
  uint32_t rev0 = kIdMax, rev1 = kIdMax;
  int m;
  if (deg <= (uint64_t)room) {
    m = (int)deg;
    if (lane < m) rev0 = (uint32_t)csr[beg + lane];
    if (lane + kWave < m) rev1 = (uint32_t)csr[beg + kWave + lane];
  } else {
    m = room;
    uint64_t best0 = kKeyMax, best1 = kKeyMax;  // the 128 smallest keys so far, ascending
    for (uint64_t c = 0; c < deg; c += kWave) {
      uint64_t key = kKeyMax;
      if (c + lane < deg) {
        const uint32_t s = (uint32_t)csr[beg + c + lane];
        key = ((hash3(base, (uint32_t)v, s, iter) >> 32) << 32) | (uint64_t)s;
      }
      key = wave_sort(key, lane);
      merge128(best0, best1, key, lane);
    }
    if (lane < room) rev0 = (uint32_t)best0;
    if (lane + kWave < room) rev1 = (uint32_t)best1;
  }
  // forward samples first, the chosen candidates behind them: object i of that
  // sequence in lane i % 64 of register i / 64
  const int total = nf + m;  // <= 2p <= 128
  const int j0 = lane - nf, j1 = lane + kWave - nf;  // positions among the candidates
  const uint32_t a0 = __shfl(rev0, j0 < 0 ? 0 : j0, kWave);
  const uint32_t b0 = __shfl(rev0, j1 & 63, kWave), b1 = __shfl(rev1, j1 & 63, kWave);
  uint32_t v0 = lane < nf ? fwd_raw : a0;
  uint32_t v1 = j1 < kWave ? b0 : b1;
  if (lane >= total) v0 = kIdMax;
  if (lane + kWave >= total) v1 = kIdMax;
  sort128(v0, v1, lane);
  const uint32_t p0 = __shfl_up(v0, 1, kWave);
  const uint32_t last0 = __shfl(v0, kWave - 1, kWave);
  uint32_t p1 = __shfl_up(v1, 1, kWave);
  if (lane == 0) p1 = last0;
  const bool keep0 = v0 != kIdMax && (lane == 0 || v0 != p0);
  const bool keep1 = v1 != kIdMax && v1 != p1;
  const uint64_t m0 = __ballot(keep0), m1 = __ballot(keep1);
  const int c0 = __popcll(m0), count = c0 + __popcll(m1);
  if (keep0) list[__popcll(m0 & lanes_below(lane))] = (int32_t)v0;
  if (keep1) list[c0 + __popcll(m1 & lanes_below(lane))] = (int32_t)v1;
  if (lane >= count && lane < 2 * p) list[lane] = -1;
  if (lane + kWave >= count && lane + kWave < 2 * p) list[lane + kWave] = -1;
  return count;
}

// One wavefront finishes both sample lists of a node (the long-list form of k_rev_select).
__global__ __launch_bounds__(kLB) void k_rev_select_long(
    int64_t n, int p, uint64_t base_new, uint64_t base_old, uint32_t iter, int32_t* snew,
    int32_t* sold, int32_t* cnew, int32_t* cold, const uint64_t* roff_new,
    const uint64_t* roff_old, const int32_t* csr_new, const int32_t* csr_old, uint32_t* capn,
    uint32_t* capo, uint32_t per_new, uint32_t per_old, uint64_t* counters) {
  const int64_t v = block_linear() * kWavesPerLB + wave_id();
  if (v >= n) return;
  const int lane = lane_id();
  const int L = 2 * p;
  int32_t* list_n = snew + v * L;
  int32_t* list_o = sold + v * L;
  const int nfn = cnew[v], nfo = cold[v];  // forward parts: at most p <= 64 entries
  const uint64_t bn = roff_new[v], dn = roff_new[v + 1] - bn;
  const uint64_t bo = roff_old[v], dO = roff_old[v + 1] - bo;
  const uint32_t rown = lane < nfn ? (uint32_t)list_n[lane] : kIdMax;
  const uint32_t rowo = lane < nfo ? (uint32_t)list_o[lane] : kIdMax;
  const int cn = select_list_long(v, p, base_new, iter, list_n, rown, nfn, csr_new, bn, dn, lane);
  const int co = select_list_long(v, p, base_old, iter, list_o, rowo, nfo, csr_old, bo, dO, lane);
  if (lane == 0) {
    cnew[v] = cn;
    cold[v] = co;
    counter_add_long(counters, C_SUMNEW, v, (uint64_t)cn);
    counter_add_long(counters, C_SUMOLD, v, (uint64_t)co);
    // bound of the results v can receive: per join it takes part in, two as a NEW sample
    // and one as an OLD sample; it takes part in at most (candidates + forward samples) joins
    capn[v] = (uint32_t)(per_new * (dn + (uint64_t)nfn));
    capo[v] = (uint32_t)(per_old * (dO + (uint64_t)nfo));
  }
}

// ---------------------------------------------------------------------------
constexpr int kLC = 64;        // dimensions per staged chunk
constexpr int kLLD = kLC + 4;  // LDS row stride (elements)
constexpr int kMaxList = 128;  // longest sample list

template <typename ACC>
__device__ inline void stage_long(ACC* dst, const float* src, int d, int d0, int part) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int j = d0 + part * 4 + q;
    dst[part * 4 + q] = (src != nullptr && j < d) ? (ACC)src[j] : (ACC)0;
  }
}
template <typename ACC>
__device__ inline void stage_long(ACC* dst, const uint8_t* src, int d, int d0, int part) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int j = d0 + part * 4 + q;
    dst[part * 4 + q] = (src != nullptr && j < d) ? (ACC)src[j] : (ACC)0;
  }
}

// One node per workgroup.  Rows of a block pair are NEW samples 64*rb.., columns are
// NEW samples 64*cb.. (cb <= rb) or OLD samples; a thread of the 16 x 16 grid holds rows
// ty + 16 r and columns tx + 16 c (r, c < 4) of the 64 x 64 block.  Per sample the
// nearest other NEW sample, the nearest OLD sample and per OLD sample the nearest NEW
// sample are kept as 64-bit keys (distance code, partner id) in LDS, so equal distances
// resolve to the smaller id whatever the order of the reductions.
template <int METRIC>
__global__ __launch_bounds__(kLB) void k_join_long(
    VecSrc vs, int64_t n, int p, int merge_mode, const int32_t* __restrict__ snew,
    const int32_t* __restrict__ sold, const int32_t* __restrict__ cnew,
    const int32_t* __restrict__ cold, const NodeMeta* __restrict__ meta, uint64_t* pslot,
    uint64_t slots, uint64_t* __restrict__ bins, uint64_t* counters) {
  using TR = JoinTraits<METRIC>;
  using T = typename TR::elem;
  using ACC = typename TR::acc;
  constexpr bool kNorms = METRIC == kCosineF32;
  __shared__ __attribute__((aligned(16))) ACC rows_t[64 * kLLD];
  __shared__ __attribute__((aligned(16))) ACC cols_t[64 * kLLD];
  __shared__ int32_t ids[2 * kMaxList];      // NEW 0..127, OLD 128..255 (-1 = none)
  __shared__ float norms_s[2 * kMaxList];    // squared norms of the samples (cosine only)
  __shared__ uint64_t nearest[3 * kMaxList]; // NEW->NEW, NEW->OLD, OLD->NEW
  __shared__ uint32_t pair_count;

  const int64_t s = block_linear();
  if (s >= n) return;
  const int tid = threadIdx.x, lane = tid & 63;
  const int L = 2 * p;
  const int nn = cnew[s], no = cold[s];
  // thread t answers for NEW sample t (t < 128) or OLD sample t - 128
  int32_t self = -1;
  if (tid < kMaxList) {
    if (tid < nn) self = snew[s * L + tid];
  } else if (tid - kMaxList < no) {
    self = sold[s * L + tid - kMaxList];
  }
  const uint32_t kth_self = self >= 0 ? meta[self].kth : 0u;
  ids[tid] = self;
  if (kNorms) norms_s[tid] = self >= 0 ? vs.norms[self] : 0.f;
  for (int i = tid; i < 3 * kMaxList; i += kLB) nearest[i] = kKeyMax;
  if (tid == 0) pair_count = 0;
  const bool do_nn = !merge_mode && nn > 1;
  if (nn == 0 || (!do_nn && no == 0)) return;  // nothing to evaluate (uniform)
  __syncthreads();

  const int tx = tid & 15, ty = tid >> 4;
  const int d = vs.d;
  const int64_t split = vs.split;
  const int row_blocks = (nn + 63) >> 6, old_blocks = (no + 63) >> 6;
  uint32_t pairs = 0;  // NEW x OLD pairs that count as evaluated, seen by this thread

  for (int rb = 0; rb < row_blocks; ++rb) {
    // column blocks: NEW blocks 0..rb (cb < 2), then the OLD blocks (cb = 2, 3)
    for (int cb = 0; cb < 4; ++cb) {
      const bool new_cols = cb < 2;
      if (new_cols ? (!do_nn || cb > rb) : (cb - 2 >= old_blocks)) continue;  // uniform
      const int row0 = 64 * rb;                                   // index into ids[]
      const int col0 = new_cols ? 64 * cb : kMaxList + 64 * (cb - 2);
      const bool diagonal = new_cols && cb == rb;
      // sub-blocks of 16 rows / 16 columns beyond the lists' ends are switched off (uniform)
      const int rows_here = nn - 64 * rb < 64 ? nn - 64 * rb : 64;
      const int cols_total = new_cols ? nn - 64 * cb : no - 64 * (cb - 2);
      const int cols_here = cols_total < 64 ? cols_total : 64;
      const int RB = (rows_here + 15) >> 4, CB = (cols_here + 15) >> 4;
      ACC acc[4][4];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = 0;
      for (int d0 = 0; d0 < d; d0 += kLC) {
        // stage the row vectors and the column vectors: 16 threads per vector, 16 vectors per pass
        const int part = tid & 15;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
          const int r = pass * 16 + (tid >> 4);
          if (pass < RB) {
            const int32_t idr = ids[row0 + r];
            stage_long<ACC>(rows_t + r * kLLD, idr >= 0 ? vs.row<T>((uint32_t)idr) : nullptr, d,
                            d0, part);
          }
          if (pass < CB) {
            const int32_t idc = ids[col0 + r];
            stage_long<ACC>(cols_t + r * kLLD, idc >= 0 ? vs.row<T>((uint32_t)idc) : nullptr, d,
                            d0, part);
          }
        }
        __syncthreads();
        const int width = (d - d0) < kLC ? (d - d0) : kLC;
        const int nsub = (width + 15) >> 4;
        for (int sub = 0; sub < nsub; ++sub) {
          // 16 dimensions at a time; dimensions past the vectors' end are staged as zeros,
          // and a pair of zeros leaves every metric's running sum as it is
          ACC a[4][16];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (r < RB) {
              const ACC* src = rows_t + (ty + 16 * r) * kLLD + sub * 16;
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int4 w = *reinterpret_cast<const int4*>(src + q * 4);
                a[r][q * 4 + 0] = __builtin_bit_cast(ACC, w.x);
                a[r][q * 4 + 1] = __builtin_bit_cast(ACC, w.y);
                a[r][q * 4 + 2] = __builtin_bit_cast(ACC, w.z);
                a[r][q * 4 + 3] = __builtin_bit_cast(ACC, w.w);
              }
            }
          }
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            if (c < CB) {
              const ACC* src = cols_t + (tx + 16 * c) * kLLD + sub * 16;
              ACC b[16];
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int4 w = *reinterpret_cast<const int4*>(src + q * 4);
                b[q * 4 + 0] = __builtin_bit_cast(ACC, w.x);
                b[q * 4 + 1] = __builtin_bit_cast(ACC, w.y);
                b[q * 4 + 2] = __builtin_bit_cast(ACC, w.z);
                b[q * 4 + 3] = __builtin_bit_cast(ACC, w.w);
              }
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                if (r < RB) {
#pragma unroll
                  for (int j = 0; j < 16; ++j) TR::step(a[r][j], b[j], acc[r][c]);
                }
              }
            }
          }
        }
        __syncthreads();
      }
      // nearest partners from the register tile
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (r >= RB) continue;
        const int R = row0 + ty + 16 * r;
        const int32_t idr = ids[R];
        uint64_t along = kKeyMax;  // nearest column object of row R in this block
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (c >= CB) continue;
          const int C = col0 + tx + 16 * c;
          const int32_t idc = ids[C];
          bool ok = idr >= 0 && idc >= 0;
          if (new_cols) {
            ok = ok && R != C;  // a diagonal block holds both orders of a pair
          } else {
            ok = ok && idc != idr;
            if (merge_mode) ok = ok && (((int64_t)idr < split) != ((int64_t)idc < split));
          }
          if (!ok) continue;
          const uint64_t code = (uint64_t)TR::code(acc[r][c], kNorms ? norms_s[R] : 0.f,
                                                   kNorms ? norms_s[C] : 0.f) << 32;
          along = vmin(along, code | (uint32_t)idc);
          if (!new_cols) {
            ++pairs;
            atomicMin(reinterpret_cast<unsigned long long*>(&nearest[2 * kMaxList + (C - kMaxList)]),
                      (unsigned long long)(code | (uint32_t)idr));
          } else if (!diagonal) {  // the pair's other direction: column object towards row object
            atomicMin(reinterpret_cast<unsigned long long*>(&nearest[C]),
                      (unsigned long long)(code | (uint32_t)idr));
          }
        }
        if (along != kKeyMax)
          atomicMin(reinterpret_cast<unsigned long long*>(&nearest[(new_cols ? 0 : kMaxList) + R]),
                    (unsigned long long)along);
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) pairs += __shfl_xor(pairs, off, kWave);
  if (lane == 0 && pairs) atomicAdd(&pair_count, pairs);
  __syncthreads();

  // hand the results on: one returning add on the destination's slot word yields the
  // segment start and this result's place in it
  uint32_t n_found = 0, n_pass = 0, n_over = 0;
  auto hand_on = [&](uint64_t key) {
    if (key == kKeyMax) return;
    ++n_found;
    if ((uint32_t)(key >> 32) > kth_self) return;  // cannot enter the destination list
    ++n_pass;
    const uint64_t w = atomicAdd(reinterpret_cast<unsigned long long*>(&pslot[self]), 1ull);
    const uint64_t at = (w >> kSlotCountBits) + (w & kSlotCountMask);
    if (at < slots) bins[at] = make_entry((uint32_t)(key >> 32), (uint32_t)key, 3u);
    else ++n_over;
  };
  if (self >= 0) {
    if (tid < kMaxList) {
      hand_on(nearest[tid]);
      hand_on(nearest[kMaxList + tid]);
    } else {
      hand_on(nearest[2 * kMaxList + tid - kMaxList]);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    n_found += __shfl_xor(n_found, off, kWave);
    n_pass += __shfl_xor(n_pass, off, kWave);
    n_over += __shfl_xor(n_over, off, kWave);
  }
  if (lane == 0) {
    if (n_pass) counter_add_long(counters, C_PASSED, s, n_pass);
    if (n_over) counter_add_long(counters, C_OVERFLOW, s, n_over);
    if (n_found) counter_add_long(counters, C_PROPS, s, n_found);
    if (tid == 0) {
      const uint64_t ev = (uint64_t)pair_count + (do_nn ? (uint64_t)nn * (nn - 1) / 2 : 0);
      if (ev) counter_add_long(counters, C_EVALS, s, ev);
    }
  }
}

}  // namespace

hipError_t launch_rev_select_long(const Shape& sh, const DevState& ds, uint64_t seed,
                                  uint32_t iter, hipStream_t st) {
  const dim3 grid = grid_blocks((sh.n + kWavesPerLB - 1) / kWavesPerLB);
  k_rev_select_long<<<grid, kLB, 0, st>>>(
      sh.n, sh.p, hash_base(seed, kTagRevNew), hash_base(seed, kTagRevOld), iter, ds.snew, ds.sold,
      ds.cnew, ds.cold, ds.roff_new, ds.roff_old, ds.csr_new, ds.csr_old, ds.capn, ds.capo,
      (uint32_t)sh.slots_new_per_appearance(), (uint32_t)sh.slots_old_per_appearance(),
      ds.counters);
  return hipGetLastError();
}

hipError_t launch_join_long(const Shape& sh, const DevState& ds, bool merge_mode, hipStream_t st) {
  VecSrc vs{sh.vec_a, sh.vec_b, sh.split, sh.d, sh.norms};
  const dim3 grid = grid_blocks(sh.n);
  const uint64_t slots = (uint64_t)sh.slots();
  const int mm = merge_mode ? 1 : 0;
#define GNND_LONG_ARGS vs, sh.n, sh.p, mm, ds.snew, ds.sold, ds.cnew, ds.cold, ds.meta, ds.pslot, \
                       slots, ds.bins, ds.counters
  switch (sh.metric) {
    case kL2F32: k_join_long<kL2F32><<<grid, kLB, 0, st>>>(GNND_LONG_ARGS); break;
    case kAngularF32: k_join_long<kAngularF32><<<grid, kLB, 0, st>>>(GNND_LONG_ARGS); break;
    case kChi2F32: k_join_long<kChi2F32><<<grid, kLB, 0, st>>>(GNND_LONG_ARGS); break;
    case kCosineF32: k_join_long<kCosineF32><<<grid, kLB, 0, st>>>(GNND_LONG_ARGS); break;
    default: k_join_long<kL2U8><<<grid, kLB, 0, st>>>(GNND_LONG_ARGS);
  }
#undef GNND_LONG_ARGS
  return hipGetLastError();
}

}  // namespace gnnd
