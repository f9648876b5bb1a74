// Cross-matching (Sec. 4.2) and selective nearest-object search (Sec. 4.3,
// Alg. 2) for one node per workgroup, canonical arithmetic: every distance is
// accumulated per pair, one fused multiply-add per dimension in dimension
// order (exact int32 for bytes), so results are bit-identical to a sequential
// evaluation.
//
// Layout: the node's <= 64 NEW and <= 64 OLD sample vectors are staged through
// LDS in chunks of 64 dimensions (coalesced row reads from HBM); the 64 x 128
// block of distances [NEW x (NEW | OLD)] is register-tiled 4 x 8 per thread
// over a 16 x 16 thread grid with the rows/columns of a thread 16 apart, so
// partially filled lists switch whole 16 x 16 sub-blocks off uniformly.  Only
// the lower block triangle of NEW x NEW is evaluated.  Per sample the nearest
// other NEW sample, the nearest OLD sample, and per OLD sample the nearest NEW
// sample are reduced straight from the register tiles; three wavefronts, one
// lane per sample, hand the results on.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

constexpr int kJB = 256;      // threads per workgroup
constexpr int kDC = 64;       // dimensions per staged chunk
constexpr int kLD = kDC + 4;  // LDS row stride (elements), keeps 16-byte alignment
constexpr int kDLD = 129;     // row stride of the distance matrix in LDS

// Stage dimensions [d0, d0 + kDC) of one vector into an LDS row (as the
// accumulation type), zero beyond the vector's end.  16 threads per row.
template <typename ACC>
__device__ inline void stage_row(ACC* dst, const float* src, int d, int d0, int part,
                                 bool aligned) {
  const int j = d0 + part * 4;
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (src != nullptr) {
    if (aligned && j + 3 < d) {
      v = *reinterpret_cast<const float4*>(src + j);
    } else {
      if (j + 0 < d) v.x = src[j + 0];
      if (j + 1 < d) v.y = src[j + 1];
      if (j + 2 < d) v.z = src[j + 2];
      if (j + 3 < d) v.w = src[j + 3];
    }
  }
  *reinterpret_cast<float4*>(dst + part * 4) = v;
}
template <typename ACC>
__device__ inline void stage_row(ACC* dst, const uint8_t* src, int d, int d0, int part,
                                 bool aligned) {
  const int j = d0 + part * 4;
  int4 v = make_int4(0, 0, 0, 0);
  if (src != nullptr) {
    if (aligned && j + 3 < d) {
      uint32_t w = *reinterpret_cast<const uint32_t*>(src + j);
      v = make_int4((int)(w & 0xff), (int)((w >> 8) & 0xff), (int)((w >> 16) & 0xff),
                    (int)(w >> 24));
    } else {
      if (j + 0 < d) v.x = src[j + 0];
      if (j + 1 < d) v.y = src[j + 1];
      if (j + 2 < d) v.z = src[j + 2];
      if (j + 3 < d) v.w = src[j + 3];
    }
  }
  *reinterpret_cast<int4*>(dst + part * 4) = v;
}

// ALL: every evaluated pair is proposed to both of its objects (the ablation
// variant without the selective update of Sec. 4.3) instead of only the nearest
// partner per sample.
template <int METRIC, bool ALL>
__global__ __launch_bounds__(kJB) void k_join_valu(
    VecSrc vs, int64_t n, int p, int merge_mode, const int32_t* __restrict__ snew,
    const int32_t* __restrict__ sold, const int32_t* __restrict__ cnew,
    const int32_t* __restrict__ cold, const NodeMeta* __restrict__ meta, uint64_t* pslot,
    uint64_t slots, uint64_t* __restrict__ bins, uint64_t* counters) {
  using TR = JoinTraits<METRIC>;
  using T = typename TR::elem;
  using ACC = typename TR::acc;
  __shared__ __attribute__((aligned(16))) ACC tile[128 * kLD];
  __shared__ int32_t ids[128];
  // per sample the nearest partner: NEW towards NEW, NEW towards OLD, OLD towards NEW
  __shared__ uint64_t nearest[192];
  __shared__ uint32_t pair_count;
  __shared__ float norms_s[128];  // squared norms of the samples (cosine only)
  constexpr bool kNorms = METRIC == kCosineF32;
  static_assert(128 * kLD >= 64 * kDLD, "distance matrix must fit in the staging tile");

  const int64_t s = block_linear();
  if (s >= n) return;  // a folded grid may be longer than the node list
  const int tid = threadIdx.x;
  const int L = 2 * p;
  const int wave = tid >> 6, lane = tid & 63;
  // Wavefronts 0 and 1 each hold the NEW sample, wavefront 2 the OLD sample, one
  // object per lane; these lanes later hand on that object's result, so the
  // threshold of its list is requested now and arrives behind the staging.
  int32_t self = -1;
  if (wave < 3 && lane < L) self = (wave < 2 ? snew : sold)[s * L + lane];
  const int nn = cnew[s], no = cold[s];
  if (lane >= (wave < 2 ? nn : no)) self = -1;
  // nothing farther than the last entry of the destination list can enter it
  const uint32_t kth_self = self >= 0 ? meta[self].kth : 0u;
  if (wave == 0) ids[lane] = self;
  else if (wave == 2) ids[64 + lane] = self;
  if (kNorms && (wave == 0 || wave == 2))
    norms_s[(wave == 0 ? 0 : 64) + lane] = self >= 0 ? vs.norms[self] : 0.f;
  if (!ALL) {
    if (tid < 192) nearest[tid] = kKeyMax;
    if (tid == 0) pair_count = 0;
  }
  const bool do_nn = !merge_mode && nn > 1;
  if (nn == 0 || (!do_nn && no == 0)) return;  // nothing to evaluate
  __syncthreads();

  const int tx = tid & 15, ty = tid >> 4;
  const int RB = (nn + 15) >> 4;  // active 16-row blocks (NEW)
  const int CO = (no + 15) >> 4;  // active 16-column blocks (OLD)
  const int d = vs.d;
  const bool aligned = (d & 3) == 0;

  ACC acc[4][8];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[r][c] = 0;

  for (int d0 = 0; d0 < d; d0 += kDC) {
    // stage: 16 threads per row, 16 rows per pass
    const int part = tid & 15;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int row = pass * 16 + (tid >> 4);
      const bool wanted = row < 64 ? (row < RB * 16) : (row - 64 < CO * 16);
      if (wanted) {
        const int32_t id = ids[row];
        const T* src = id >= 0 ? vs.row<T>((uint32_t)id) : nullptr;
        stage_row<ACC>(tile + row * kLD, src, d, d0, part, aligned);
      }
    }
    __syncthreads();
    const int width = (d - d0) < kDC ? (d - d0) : kDC;
    const int nsub = (width + 15) >> 4;
    for (int sub = 0; sub < nsub; ++sub) {
      ACC a[4][16];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (r < RB) {
          const ACC* src = tile + (ty + 16 * r) * kLD + sub * 16;
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
      for (int c = 0; c < 8; ++c) {
        const bool col_on = c < 4 ? (do_nn && c < RB) : (c - 4 < CO);
        if (col_on) {
          const int crow = c < 4 ? (tx + 16 * c) : (64 + tx + 16 * (c - 4));
          const ACC* src = tile + crow * kLD + sub * 16;
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
            if (r < RB && (c >= 4 || c <= r)) {
#pragma unroll
              for (int j = 0; j < 16; ++j) TR::step(a[r][j], b[j], acc[r][c]);
            }
          }
        }
      }
    }
    __syncthreads();
  }

  const int64_t split = vs.split;
  uint32_t* Dm = reinterpret_cast<uint32_t*>(tile);
  if constexpr (ALL) {
    // distances (as order-preserving codes) to LDS: Dm[row][col], col < 64 NEW, >= 64 OLD
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const bool on = r < RB && (c < 4 ? (do_nn && c <= r) : (c - 4 < CO));
        if (on) {
          const int col = c < 4 ? (tx + 16 * c) : (64 + tx + 16 * (c - 4));
          Dm[(ty + 16 * r) * kDLD + col] =
              TR::code(acc[r][c], kNorms ? norms_s[ty + 16 * r] : 0.f, kNorms ? norms_s[col] : 0.f);
        }
      }
  } else {
    // Nearest-object search straight from the register tiles.  A thread holds
    // rows R = ty + 16r and columns tx + 16c: the minimum along a row is
    // completed over the 16 lanes that share ty, the minimum along a column
    // over the lanes of the wavefront that share tx and then over the four
    // wavefronts through LDS.  Keys are (distance code, partner id), so equal
    // distances resolve to the smaller id whatever the order of reduction.
    int32_t idc[8];
    float normc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      idc[c] = ids[c < 4 ? (tx + 16 * c) : (64 + tx + 16 * (c - 4))];
      normc[c] = kNorms ? norms_s[c < 4 ? (tx + 16 * c) : (64 + tx + 16 * (c - 4))] : 0.f;
    }
    uint64_t down[8];  // per column: nearest row object seen by this thread
#pragma unroll
    for (int c = 0; c < 8; ++c) down[c] = kKeyMax;
    uint32_t pairs = 0;  // NEW x OLD pairs that count as evaluated
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (r < RB) {  // uniform over the workgroup
        const int R = ty + 16 * r;
        const int32_t idr = ids[R];
        uint64_t to_new = kKeyMax, to_old = kKeyMax;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const bool on = c < 4 ? (do_nn && c <= r) : (c - 4 < CO);
          if (!on) continue;
          const int32_t other = idc[c];
          bool ok = idr >= 0 && other >= 0;
          if (c < 4) {
            ok = ok && (c < r || tx != ty);  // the diagonal block holds both orders of a pair
          } else {
            ok = ok && other != idr;
            if (merge_mode) ok = ok && (((int64_t)idr < split) != ((int64_t)other < split));
          }
          if (!ok) continue;
          const uint64_t code = (uint64_t)TR::code(acc[r][c], kNorms ? norms_s[R] : 0.f,
                                                   kNorms ? normc[c] : 0.f) << 32;
          const uint64_t here = code | (uint32_t)other, there = code | (uint32_t)idr;
          if (c < 4) {
            to_new = vmin(to_new, here);
            if (c < r) down[c] = vmin(down[c], there);
          } else {
            ++pairs;
            to_old = vmin(to_old, here);
            down[c] = vmin(down[c], there);
          }
        }
#pragma unroll
        for (int j = 1; j < 16; j <<= 1) {
          to_new = vmin(to_new, xor_lanes(to_new, j, lane));
          to_old = vmin(to_old, xor_lanes(to_old, j, lane));
        }
        if (tx == 0) {
          if (to_new != kKeyMax) atomicMin(reinterpret_cast<unsigned long long*>(&nearest[R]),
                                           (unsigned long long)to_new);
          if (to_old != kKeyMax) nearest[64 + R] = to_old;  // rows have one writer
        }
      }
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const bool on = c < 4 ? (do_nn && c + 1 < RB) : (c - 4 < CO);
      if (on) {  // uniform over the workgroup
        uint64_t v = down[c];
        v = vmin(v, xor_lanes(v, 16, lane));
        v = vmin(v, xor_lanes(v, 32, lane));
        if (ty == (wave << 2) && v != kKeyMax)
          atomicMin(reinterpret_cast<unsigned long long*>(
                        &nearest[c < 4 ? (tx + 16 * c) : (128 + tx + 16 * (c - 4))]),
                    (unsigned long long)v);
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) pairs += __shfl_xor(pairs, off, kWave);
    if (lane == 0 && pairs) atomicAdd(&pair_count, pairs);
  }
  __syncthreads();

  // wave 0: NEW samples towards NEW, wave 1: NEW towards OLD, wave 2: OLD towards NEW
  if (wave > 2) return;
  uint64_t best = kKeyMax;
  uint32_t evaluated = 0;
  uint32_t n_found = 0, n_pass = 0, n_over = 0;  // this lane's results
  if (wave == 0 && !do_nn) self = -1;
  // hand a result to the destination's segment of the proposal array: one
  // returning add yields the segment start and this result's place in it
  auto hand_on = [&](uint64_t key) {
    ++n_found;
    if ((uint32_t)(key >> 32) > kth_self) return;  // dropped here already
    ++n_pass;
    const uint64_t w = atomicAdd(reinterpret_cast<unsigned long long*>(&pslot[self]), 1ull);
    const uint64_t at = (w >> kSlotCountBits) + (w & kSlotCountMask);
    if (at < slots) bins[at] = make_entry((uint32_t)(key >> 32), (uint32_t)key, 3u);
    else ++n_over;
  };
  if constexpr (ALL) {
    if (wave == 0) {
      if (self >= 0) {
        for (int v = 0; v < nn; ++v) {
          if (v == lane) continue;
          const uint32_t code = ((v >> 4) <= (lane >> 4)) ? Dm[lane * kDLD + v] : Dm[v * kDLD + lane];
          hand_on(((uint64_t)code << 32) | (uint32_t)ids[v]);
        }
      }
    } else if (wave == 1) {
      if (self >= 0) {
        for (int o = 0; o < no; ++o) {
          const int32_t other = ids[64 + o];
          bool ok = other != self;
          if (merge_mode) ok = ok && (((int64_t)self < split) != ((int64_t)other < split));
          if (!ok) continue;
          ++evaluated;
          hand_on(((uint64_t)Dm[lane * kDLD + 64 + o] << 32) | (uint32_t)other);
        }
      }
    } else {
      if (self >= 0) {
        for (int u = 0; u < nn; ++u) {
          const int32_t other = ids[u];
          bool ok = other != self;
          if (merge_mode) ok = ok && (((int64_t)self < split) != ((int64_t)other < split));
          if (!ok) continue;
          hand_on(((uint64_t)Dm[u * kDLD + 64 + lane] << 32) | (uint32_t)other);
        }
      }
    }
  } else {
    if (self >= 0) best = nearest[wave * 64 + lane];
    if (wave == 1 && lane == 0) evaluated = pair_count;
  }
  if (!ALL && best != kKeyMax) hand_on(best);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    n_found += __shfl_xor(n_found, off, kWave);
    n_pass += __shfl_xor(n_pass, off, kWave);
    n_over += __shfl_xor(n_over, off, kWave);
    evaluated += __shfl_xor(evaluated, off, kWave);
  }
  if (lane == 0) {
    uint64_t* cs = counters + (s & (kStripes - 1)) * C_SLOTS;
    if (n_pass) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_PASSED),
                          (unsigned long long)n_pass);
    if (n_over) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_OVERFLOW),
                          (unsigned long long)n_over);
    if (n_found) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_PROPS),
                           (unsigned long long)n_found);
    if (wave == 1) {
      const uint64_t ev = (uint64_t)evaluated + (do_nn ? (uint64_t)nn * (nn - 1) / 2 : 0);
      if (ev) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_EVALS),
                        (unsigned long long)ev);
    }
  }
}

template <bool ALL>
static void launch_join_as(const Shape& sh, const DevState& ds, bool merge_mode, hipStream_t st) {
  VecSrc vs{sh.vec_a, sh.vec_b, sh.split, sh.d, sh.norms};
  const dim3 grid = grid_blocks(sh.n);
  const uint64_t slots = (uint64_t)sh.slots();  // size of the proposal array
  const int mm = merge_mode ? 1 : 0;
#define GNND_JOIN_ARGS vs, sh.n, sh.p, mm, ds.snew, ds.sold, ds.cnew, ds.cold, ds.meta, ds.pslot, \
                       slots, ds.bins, ds.counters
  switch (sh.metric) {
    case kL2F32: k_join_valu<kL2F32, ALL><<<grid, kJB, 0, st>>>(GNND_JOIN_ARGS); break;
    case kAngularF32: k_join_valu<kAngularF32, ALL><<<grid, kJB, 0, st>>>(GNND_JOIN_ARGS); break;
    case kChi2F32: k_join_valu<kChi2F32, ALL><<<grid, kJB, 0, st>>>(GNND_JOIN_ARGS); break;
    case kCosineF32: k_join_valu<kCosineF32, ALL><<<grid, kJB, 0, st>>>(GNND_JOIN_ARGS); break;
    default: k_join_valu<kL2U8, ALL><<<grid, kJB, 0, st>>>(GNND_JOIN_ARGS);
  }
#undef GNND_JOIN_ARGS
}

hipError_t launch_join(const Shape& sh, const DevState& ds, int path, bool merge_mode,
                       hipStream_t st) {
  (void)path;
  if (2 * sh.p > kWave) return launch_join_long(sh, ds, merge_mode, st);  // sample lists beyond 64
  if (sh.all_pairs) launch_join_as<true>(sh, ds, merge_mode, st);
  else launch_join_as<false>(sh, ds, merge_mode, st);
  return hipGetLastError();
}

}  // namespace gnnd
