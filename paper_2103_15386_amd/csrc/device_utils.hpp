// Device-side building blocks shared by the GNND kernels: the counter-based
// hash, the order-preserving distance encoding, packed list entries and the
// 64-lane sorting / merging networks that act on one value per lane.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gnnd {

constexpr int kWave = 64;
constexpr uint64_t kKeyMax = ~0ull;
constexpr uint32_t kIdMax = 0x7fffffffu;

enum : int { kL2F32 = 0, kAngularF32 = 1, kL2U8 = 2, kChi2F32 = 3, kCosineF32 = 4 };
enum : uint32_t { kTagInit = 1, kTagRevNew = 2, kTagRevOld = 3, kTagMerge = 4 };
constexpr uint32_t kHashAttempts = 256;

// ---- counter-based random numbers ---------------------------------------
// hash(seed, tag, a, b, c): three rounds of the splitmix64 output mixer over
// (seed, tag), the packed pair (a, b), and c.  Any thread can draw any number.
__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xbf58476d1ce4e5b9ull;
  z ^= z >> 27;
  z *= 0x94d049bb133111ebull;
  z ^= z >> 31;
  return z;
}
// The (seed, tag) round depends on nothing per thread: computed once on the host.
__host__ __device__ inline uint64_t hash_base(uint64_t seed, uint32_t tag) {
  return mix64(seed + 0x9e3779b97f4a7c15ull * ((uint64_t)tag + 1));
}
__device__ inline uint64_t hash3(uint64_t base, uint32_t a, uint32_t b, uint32_t c) {
  uint64_t h = mix64(base ^ (((uint64_t)a << 32) | (uint64_t)b));
  return mix64(h + (uint64_t)c);
}
// upper 32 hash bits mapped onto [0, n) by multiply-high
__device__ inline uint32_t bounded(uint64_t h, uint32_t n) {
  return __umulhi((uint32_t)(h >> 32), n);
}

// ---- distances as order-preserving 32-bit codes -------------------------
// A float (possibly negative: 1 - dot can round below zero) or an int32 maps to
// an unsigned code with the same order, so (code << 32 | id) compares like
// (distance, id).
__device__ inline uint32_t ord_f32(float x) {
  uint32_t b = __float_as_uint(x);
  return b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
}
__device__ inline float unord_f32(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : ~o);
}
__device__ inline uint32_t ord_i32(int32_t x) { return (uint32_t)x ^ 0x80000000u; }
__device__ inline int32_t unord_i32(uint32_t o) { return (int32_t)(o ^ 0x80000000u); }

// ---- packed list entry ---------------------------------------------------
// 64 bits: [63:32] distance code, [31:2] neighbour id, bit 1 "admitted by the
// update in progress", bit 0 NEW flag.  Unsigned comparison of two entries
// with different ids orders them by (distance, id).
__device__ inline uint64_t make_entry(uint32_t code, uint32_t id, uint32_t flags) {
  return ((uint64_t)code << 32) | ((uint64_t)id << 2) | flags;
}
__device__ inline uint32_t entry_id(uint64_t e) { return ((uint32_t)e) >> 2; }
__device__ inline uint32_t entry_code(uint64_t e) { return (uint32_t)(e >> 32); }
__device__ inline uint64_t entry_key(uint64_t e) { return e >> 2; }  // (distance, id) only

// ---- wavefront helpers (one value per lane, 64 lanes) --------------------
__device__ inline int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
// Number of this wavefront inside its workgroup, as a scalar: every lane holds the same
// value, and saying so keeps what is derived from it (row numbers, base addresses) in
// scalar registers.
__device__ inline int wave_id() {
  return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}
__device__ inline uint64_t lanes_below(int lane) { return (1ull << lane) - 1ull; }

// A launch may not span 2^32 threads in one grid dimension (16 M workgroups of
// 256); launches over more workgroups fold them into two dimensions, and the
// kernels number their workgroups with this.  Workgroups past the end of the
// work (the last row of the fold) must leave on their own index checks.
__device__ inline int64_t block_linear() {
  return (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
}

__device__ inline uint64_t readlane64(uint64_t x, int l) {
  uint32_t lo = __builtin_amdgcn_readlane((uint32_t)x, l);
  uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(x >> 32), l);
  return ((uint64_t)hi << 32) | lo;
}

template <typename T>
__device__ inline T vmin(T a, T b) { return a < b ? a : b; }
template <typename T>
__device__ inline T vmax(T a, T b) { return a < b ? b : a; }

// Value of lane (lane ^ j), j a power of two, without going through LDS: data
// parallel primitives inside a row of 16 lanes (quad permutes, row shifts under
// bank masks, row rotate) and the row / half swaps across rows.  `j` must be a
// compile-time constant after unrolling.
__device__ inline uint32_t xor_lanes(uint32_t v, int j, int lane) {
  switch (j) {
    case 1: return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // quad_perm:[1,0,3,2]
    case 2: return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);  // quad_perm:[2,3,0,1]
    case 4: {
      // lanes 0-3 and 8-11 of a row read 4 lanes up (row_shl:4), the others 4 lanes down (row_shr:4)
      int r = __builtin_amdgcn_update_dpp(0, (int)v, 0x104, 0xF, 0x5, false);
      r = __builtin_amdgcn_update_dpp(r, (int)v, 0x114, 0xF, 0xA, false);
      return (uint32_t)r;
    }
    case 8: return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xF, 0xF, true);  // row_ror:8
    case 16: {
      // rows 1 and 3 of the first copy change places with rows 0 and 2 of the second
      auto sw = __builtin_amdgcn_permlane16_swap(v, v, false, false);
      return (lane & 16) ? sw[0] : sw[1];
    }
    default: {
      // the upper half of the first copy changes places with the lower half of the second
      auto sw = __builtin_amdgcn_permlane32_swap(v, v, false, false);
      return (lane & 32) ? sw[0] : sw[1];
    }
  }
}
__device__ inline uint64_t xor_lanes(uint64_t v, int j, int lane) {
  const uint32_t lo = xor_lanes((uint32_t)v, j, lane);
  const uint32_t hi = xor_lanes((uint32_t)(v >> 32), j, lane);
  return ((uint64_t)hi << 32) | lo;
}

// Value of lane 63 - lane: mirror inside the row, then swap rows and halves.
__device__ inline uint32_t reverse_lanes(uint32_t v, int lane) {
  const uint32_t m = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x140, 0xF, 0xF, true);  // row_mirror
  return xor_lanes(xor_lanes(m, 16, lane), 32, lane);
}
__device__ inline uint64_t reverse_lanes(uint64_t v, int lane) {
  const uint32_t lo = reverse_lanes((uint32_t)v, lane);
  const uint32_t hi = reverse_lanes((uint32_t)(v >> 32), lane);
  return ((uint64_t)hi << 32) | lo;
}

// One compare-exchange of a sorting network: this lane keeps the smaller of
// its value and its partner's when keep_min, else the larger.  (Equal values:
// either.)  One comparison; the lane pattern keep_min folds into the mask.
template <typename T>
__device__ inline T exchange(T v, T o, bool keep_min) {
  return ((o < v) == keep_min) ? o : v;
}
// 32-bit values: min and max can take the partner straight from the lane
// permutation (no separate move), then one select on the lane pattern.
__device__ inline uint32_t exchange(uint32_t v, uint32_t o, bool keep_min) {
  const uint32_t lo = v < o ? v : o, hi = v < o ? o : v;
  return keep_min ? lo : hi;
}

// Full ascending sort of 64 lane values (bitonic network, 21 exchange stages).
template <typename T>
__device__ inline T wave_sort(T v, int lane) {
#pragma unroll
  for (int k = 2; k <= kWave; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      const T o = xor_lanes(v, j, lane);
      v = exchange(v, o, ((lane & j) == 0) == ((lane & k) == 0));
    }
  }
  return v;
}

// Ascending sort when only the first `count` lanes hold real values and all
// other lanes hold the maximum: the network over the next power of two is
// enough (short lists are the common case), the tail is in place already.
template <int N, typename T>
__device__ inline T wave_sort_first(T v, int lane) {
#pragma unroll
  for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      const T o = xor_lanes(v, j, lane);
      v = exchange(v, o, ((lane & j) == 0) == ((lane & k) == 0));
    }
  }
  return v;
}
template <typename T>
__device__ inline T wave_sort_upto(T v, int lane, int count) {
  if (count <= 1) return v;
  if (count <= 2) return wave_sort_first<2>(v, lane);
  if (count <= 4) return wave_sort_first<4>(v, lane);
  if (count <= 8) return wave_sort_first<8>(v, lane);
  if (count <= 16) return wave_sort_first<16>(v, lane);
  if (count <= 32) return wave_sort_first<32>(v, lane);
  return wave_sort(v, lane);
}

// Lanes hold a bitonic sequence (ascending then descending, or an element-wise
// min of an ascending and a reversed ascending one): 6 stages sort it ascending.
template <typename T>
__device__ inline T wave_bitonic_merge(T v, int lane) {
#pragma unroll
  for (int j = kWave >> 1; j > 0; j >>= 1) {
    const T o = xor_lanes(v, j, lane);
    v = exchange(v, o, (lane & j) == 0);
  }
  return v;
}

// The 64 smallest of two ascending 64-lane sequences, ascending.
template <typename T>
__device__ inline T wave_merge_smallest(T a_sorted, T b_sorted, int lane) {
  const T br = reverse_lanes(b_sorted, lane);
  return wave_bitonic_merge(vmin(a_sorted, br), lane);
}

// 128 values, two per lane (value i in lane i % 64 of register i / 64), ascending over
// (lo, hi): two 64-lane networks and a 128-wide bitonic merge.
template <typename T>
__device__ inline void sort128(T& lo, T& hi, int lane) {
  lo = wave_sort(lo, lane);
  hi = wave_sort(hi, lane);
  const T t = reverse_lanes(hi, lane);  // lo ++ t is bitonic
  const T a = vmin(lo, t), b = vmax(lo, t);
  lo = wave_bitonic_merge(a, lane);
  hi = wave_bitonic_merge(b, lane);
}

// (lo, hi) ascending, c ascending (64 values): afterwards (lo, hi) holds the 128
// smallest of the 192, ascending (c is split against lo; the larger half goes on to hi).
template <typename T>
__device__ inline void merge128(T& lo, T& hi, T c, int lane) {
  const T t = reverse_lanes(c, lane);
  const T a = vmin(lo, t), b = vmax(lo, t);
  lo = wave_bitonic_merge(a, lane);
  const T spill = wave_bitonic_merge(b, lane);  // the 64 largest of lo and c, ascending
  hi = wave_merge_smallest(hi, spill, lane);
}

// Stable compaction of the lanes with keep == true to the front; the other
// lanes end up behind them holding `fill`.
__device__ inline uint64_t wave_compact(uint64_t v, bool keep, uint64_t fill, int lane) {
  uint64_t mask = __ballot(keep);
  int nkeep = __popcll(mask);
  int before = __popcll(mask & lanes_below(lane));
  int dst = keep ? before : nkeep + (lane - before);
  uint64_t x = keep ? v : fill;
  uint32_t lo = __builtin_amdgcn_ds_permute(dst << 2, (int)(uint32_t)x);
  uint32_t hi = __builtin_amdgcn_ds_permute(dst << 2, (int)(uint32_t)(x >> 32));
  return ((uint64_t)hi << 32) | lo;
}

// Drop from `pk` (one candidate per lane, kKeyMax = none) what cannot enter the
// ascending list `row` of k entries: not closer than its last entry, already
// in it, or a repeat of another candidate.  Returns the survivors ascending.
__device__ inline uint64_t filter_candidates(uint64_t pk, uint64_t row, int k, int lane,
                                             bool& any) {
  const uint64_t last = readlane64(row, k - 1);
  if (pk != kKeyMax && entry_key(pk) >= entry_key(last)) pk = kKeyMax;
  any = __ballot(pk != kKeyMax) != 0ull;
  if (!any) return pk;
  // already in the list?  The 64 lanes of `row` ascend (unused lanes hold the
  // maximum), so each candidate finds its lower bound in six halving steps.
  const uint64_t kk = entry_key(pk);
  int pos = 0;
#pragma unroll
  for (int step = kWave / 2; step > 0; step >>= 1) {
    const uint64_t r = __shfl(row, pos + step - 1, kWave);
    pos += (entry_key(r) < kk) ? step : 0;
  }
  if (entry_key(__shfl(row, pos, kWave)) == kk) pk = kKeyMax;
  const uint64_t left = __ballot(pk != kKeyMax);
  any = left != 0ull;
  if (!any) return pk;
  // survivors to the front, then a sorting network just wide enough for them
  pk = wave_compact(pk, pk != kKeyMax, kKeyMax, lane);
  pk = wave_sort_upto(pk, lane, __popcll(left));
  const uint64_t prev = __shfl_up(pk, 1, kWave);
  const bool rep = lane > 0 && pk != kKeyMax && entry_key(pk) == entry_key(prev);
  if (__ballot(rep) != 0ull) pk = wave_compact(pk, !rep, kKeyMax, lane);
  return pk;
}

// ---- canonical distances --------------------------------------------------
// Float metrics accumulate one fused multiply-add per dimension, in dimension
// order, in float32; bytes accumulate exact int32 squares.  The result is the
// order-preserving code of the distance.
template <int METRIC>
struct DistOf;

template <>
struct DistOf<kL2F32> {
  using elem = float;
  __device__ static uint32_t eval(const float* a, const float* b, int d) {
    float acc = 0.f;
    int j = 0;
    if ((d & 3) == 0) {
      const float4* a4 = reinterpret_cast<const float4*>(a);
      const float4* b4 = reinterpret_cast<const float4*>(b);
      for (; j < (d >> 2); ++j) {
        float4 x = a4[j], y = b4[j];
        float t;
        t = x.x - y.x; acc = __fmaf_rn(t, t, acc);
        t = x.y - y.y; acc = __fmaf_rn(t, t, acc);
        t = x.z - y.z; acc = __fmaf_rn(t, t, acc);
        t = x.w - y.w; acc = __fmaf_rn(t, t, acc);
      }
    } else {
      for (; j < d; ++j) {
        float t = a[j] - b[j];
        acc = __fmaf_rn(t, t, acc);
      }
    }
    return ord_f32(acc);
  }
};

template <>
struct DistOf<kAngularF32> {
  using elem = float;
  __device__ static uint32_t eval(const float* a, const float* b, int d) {
    float acc = 0.f;
    int j = 0;
    if ((d & 3) == 0) {
      const float4* a4 = reinterpret_cast<const float4*>(a);
      const float4* b4 = reinterpret_cast<const float4*>(b);
      for (; j < (d >> 2); ++j) {
        float4 x = a4[j], y = b4[j];
        acc = __fmaf_rn(x.x, y.x, acc);
        acc = __fmaf_rn(x.y, y.y, acc);
        acc = __fmaf_rn(x.z, y.z, acc);
        acc = __fmaf_rn(x.w, y.w, acc);
      }
    } else {
      for (; j < d; ++j) acc = __fmaf_rn(a[j], b[j], acc);
    }
    return ord_f32(1.0f - acc);
  }
};

// Chi-square distance of non-negative vectors: sum of (a - b)^2 / (a + b) over
// the dimensions with a + b > 0; every operation rounded on its own (there is no
// multiply feeding an add, so nothing can fuse), correctly rounded division.
__device__ inline float chi2_term(float a, float b, float acc) {
  const float diff = __fsub_rn(a, b), sum = __fadd_rn(a, b);
  return sum > 0.f ? __fadd_rn(acc, __fdiv_rn(__fmul_rn(diff, diff), sum)) : acc;
}
template <>
struct DistOf<kChi2F32> {
  using elem = float;
  __device__ static uint32_t eval(const float* a, const float* b, int d) {
    float acc = 0.f;
    for (int j = 0; j < d; ++j) acc = chi2_term(a[j], b[j], acc);
    return ord_f32(acc);
  }
};

// Cosine distance of vectors of any length: 1 - a.b / sqrt(|a|^2 |b|^2); a zero
// vector is at distance 1 from everything.  The inner product and the squared
// norms are accumulated like the angular inner product (a squared norm belongs
// to its vector alone, so it can be computed once and kept); product, root,
// quotient and difference are each rounded on their own.
__device__ inline uint32_t cosine_code(float dot, float na, float nb) {
  // sqrtf is the correctly rounded root (the compiler's default for HIP); the
  // intrinsic named after round-to-nearest maps to the approximate instruction
  const float den = sqrtf(__fmul_rn(na, nb));
  return ord_f32(den > 0.f ? __fsub_rn(1.0f, __fdiv_rn(dot, den)) : 1.0f);
}
template <>
struct DistOf<kCosineF32> {
  using elem = float;
  __device__ static uint32_t eval(const float* a, const float* b, int d) {
    float dot = 0.f, na = 0.f, nb = 0.f;
    for (int j = 0; j < d; ++j) {
      const float x = a[j], y = b[j];
      dot = __fmaf_rn(x, y, dot);
      na = __fmaf_rn(x, x, na);
      nb = __fmaf_rn(y, y, nb);
    }
    return cosine_code(dot, na, nb);
  }
};

template <>
struct DistOf<kL2U8> {
  using elem = uint8_t;
  __device__ static uint32_t eval(const uint8_t* a, const uint8_t* b, int d) {
    int32_t acc = 0;
    int j = 0;
    if ((d & 3) == 0) {
      const uint32_t* a4 = reinterpret_cast<const uint32_t*>(a);
      const uint32_t* b4 = reinterpret_cast<const uint32_t*>(b);
      for (; j < (d >> 2); ++j) {
        uint32_t x = a4[j], y = b4[j];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          int32_t t = (int32_t)((x >> (8 * q)) & 0xff) - (int32_t)((y >> (8 * q)) & 0xff);
          acc += t * t;
        }
      }
    } else {
      for (; j < d; ++j) {
        int32_t t = (int32_t)a[j] - (int32_t)b[j];
        acc += t * t;
      }
    }
    return ord_i32(acc);
  }
};

// Vectors may live in two arrays (the two sets of a merge): rows below `split`
// come from the first, the others from the second.
struct VecSrc {
  const void* a;
  const void* b;
  int64_t split;
  int32_t d;
  const float* norms = nullptr;  // squared norm per id where the metric needs it (cosine)
  template <typename T>
  __device__ const T* row(uint32_t id) const {
    return ((int64_t)id < split) ? reinterpret_cast<const T*>(a) + (int64_t)id * d
                                 : reinterpret_cast<const T*>(b) + ((int64_t)id - split) * d;
  }
};

// The same arithmetic one step at a time (one dimension of one pair), for the
// kernels that walk many pairs through staged chunks of dimensions.
template <int METRIC>
struct JoinTraits;
template <>
struct JoinTraits<kL2F32> {
  using elem = float;
  using acc = float;
  __device__ static void step(float a, float b, float& s) {
    float t = a - b;
    s = __fmaf_rn(t, t, s);
  }
  __device__ static uint32_t code(float s) { return ord_f32(s); }
  __device__ static uint32_t code(float s, float, float) { return code(s); }
};
template <>
struct JoinTraits<kAngularF32> {
  using elem = float;
  using acc = float;
  __device__ static void step(float a, float b, float& s) { s = __fmaf_rn(a, b, s); }
  __device__ static uint32_t code(float s) { return ord_f32(1.0f - s); }
  __device__ static uint32_t code(float s, float, float) { return code(s); }
};
// cosine: the running sum is the inner product; the squared norms of the two
// vectors come from the per-id array (VecSrc::norms)
template <>
struct JoinTraits<kCosineF32> {
  using elem = float;
  using acc = float;
  __device__ static void step(float a, float b, float& s) { s = __fmaf_rn(a, b, s); }
  __device__ static uint32_t code(float s, float na, float nb) { return cosine_code(s, na, nb); }
};
template <>
struct JoinTraits<kChi2F32> {
  using elem = float;
  using acc = float;
  __device__ static void step(float a, float b, float& s) { s = chi2_term(a, b, s); }
  __device__ static uint32_t code(float s) { return ord_f32(s); }
  __device__ static uint32_t code(float s, float, float) { return code(s); }
};
template <>
struct JoinTraits<kL2U8> {
  using elem = uint8_t;
  using acc = int32_t;
  __device__ static void step(int32_t a, int32_t b, int32_t& s) {
    int32_t t = a - b;
    s += __mul24(t, t);
  }
  __device__ static uint32_t code(int32_t s) { return ord_i32(s); }
  __device__ static uint32_t code(int32_t s, float, float) { return code(s); }
};

// Canonical distances from object s to one object per lane (`id`, meaningful
// where `on`).  The 64 rows and the row of s are staged through the wave's LDS
// tile in chunks of kEvalChunk dimensions with coalesced reads (8 lanes per row
// chunk), then every lane accumulates its own pair in dimension order: the
// arithmetic of DistOf<METRIC>::eval, without 64 lanes each walking a row of its
// own through HBM.  All 64 lanes must call it together.
constexpr int kEvalChunk = 32;
constexpr int kEvalStride = kEvalChunk + 1;  // odd stride: lanes walk their rows free of bank conflicts
constexpr int kEvalTileWords = 65 * kEvalStride;

template <int METRIC>
__device__ inline uint32_t wave_distances(const VecSrc& vs, uint32_t s, uint32_t id, bool on,
                                          uint32_t* tile_raw, int lane) {
  using TR = JoinTraits<METRIC>;
  using T = typename TR::elem;
  using ACC = typename TR::acc;
  ACC* tile = reinterpret_cast<ACC*>(tile_raw);
  const int d = vs.d;
  const bool aligned = (d & 3) == 0;
  const int part = lane & 7, rsel = lane >> 3;
  ACC acc = 0;
  for (int d0 = 0; d0 < d; d0 += kEvalChunk) {
#pragma unroll
    for (int r0 = 0; r0 < 72; r0 += 8) {  // rows 0..63: the lanes' objects, row 64: s
      const int r = r0 + rsel;
      const uint32_t rid = __shfl(id, r & 63, kWave);
      const int ron = __shfl((int)on, r & 63, kWave);
      const bool want = r < 64 ? ron != 0 : r == 64;
      if (want) {
        const T* src = vs.row<T>(r < 64 ? rid : s);
        const int j = d0 + part * 4;
        ACC v[4] = {0, 0, 0, 0};
        if (sizeof(T) == 4 && aligned && j + 3 < d) {
          const float4 f = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(src) + j);
          v[0] = (ACC)f.x; v[1] = (ACC)f.y; v[2] = (ACC)f.z; v[3] = (ACC)f.w;
        } else if (sizeof(T) == 1 && aligned && j + 3 < d) {  // four bytes in one load
          const uint32_t w = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(src) + j);
          v[0] = (ACC)(w & 0xff); v[1] = (ACC)((w >> 8) & 0xff);
          v[2] = (ACC)((w >> 16) & 0xff); v[3] = (ACC)(w >> 24);
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (j + q < d) v[q] = (ACC)src[j + q];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) tile[r * kEvalStride + part * 4 + q] = v[q];
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int width = d - d0 < kEvalChunk ? d - d0 : kEvalChunk;
    if (on)
      for (int j = 0; j < width; ++j)
        TR::step(tile[64 * kEvalStride + j], tile[lane * kEvalStride + j], acc);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if constexpr (METRIC == kCosineF32) return TR::code(acc, vs.norms[s], on ? vs.norms[id] : 0.f);
  else return TR::code(acc);
}

// Numbering inside one merge (Sec. 5.1 shards).  The two sets are the ranges
// [base1, base1 + n1) and [base2, base2 + n2) of a larger collection; inside
// the merge S1 is 0..n1-1, S2 is n1..n-1, and any other object (a list entry
// left by an earlier merge with a third shard: "frozen", never sampled) is
// n + its collection id.
struct MergeIds {
  int64_t n1, base1, n2, base2;
  __host__ __device__ uint32_t to_internal(int64_t g) const {
    if (g >= base1 && g < base1 + n1) return (uint32_t)(g - base1);
    if (g >= base2 && g < base2 + n2) return (uint32_t)(n1 + g - base2);
    return (uint32_t)(n1 + n2 + g);
  }
  __host__ __device__ int32_t to_global(int64_t i) const {
    if (i < n1) return (int32_t)(base1 + i);
    if (i < n1 + n2) return (int32_t)(base2 + i - n1);
    return (int32_t)(i - n1 - n2);
  }
};

// Draw `count` (<= 64) distinct ids out of [0, range) + base for node s, one per
// lane: slot j takes hash(base_hash, s, j, attempt) mapped onto the range for
// attempt = 0, 1, ... until the id differs from `forbid` and from the ids of
// the slots before it; after kHashAttempts failures it walks to the next free
// id cyclically.  Wave-uniform loop; returns the id of slot `lane` (lanes >=
// count: undefined).
// First attempt of slot `lane`.  When the first attempts of all slots are
// pairwise distinct and none is `forbid`, the slot-by-slot rule accepts every
// one of them as it stands (a slot only ever looks at the slots before it).
__device__ inline uint32_t draw_first(uint64_t base_hash, uint32_t s, uint32_t range,
                                      uint32_t base, int lane) {
  return bounded(hash3(base_hash, s, (uint32_t)lane, 0u), range) + base;
}
__device__ inline uint32_t draw_slot_by_slot(uint64_t base_hash, uint32_t s, int count,
                                             uint32_t range, uint32_t base, uint32_t forbid,
                                             int lane);
__device__ inline uint32_t draw_distinct(uint64_t base_hash, uint32_t s, int count,
                                         uint32_t range, uint32_t base, uint32_t forbid,
                                         int lane) {
  const uint32_t first = draw_first(base_hash, s, range, base, lane);
  bool clash_any = lane < count && first == forbid;
  for (int j = 0; j + 1 < count; ++j) {
    const uint32_t cj = (uint32_t)__builtin_amdgcn_readlane((int)first, j);
    clash_any |= lane > j && lane < count && first == cj;
  }
  if (__ballot(clash_any) == 0ull) return first;
  return draw_slot_by_slot(base_hash, s, count, range, base, forbid, lane);
}
__device__ inline uint32_t draw_slot_by_slot(uint64_t base_hash, uint32_t s, int count,
                                             uint32_t range, uint32_t base, uint32_t forbid,
                                             int lane) {
  uint32_t mine = 0xffffffffu;
  for (int j = 0; j < count; ++j) {
    uint32_t cand = 0;
    bool ok = false;
    for (uint32_t attempt = 0; attempt < kHashAttempts && !ok; ++attempt) {
      cand = bounded(hash3(base_hash, s, (uint32_t)j, attempt), range) + base;
      bool clash = (lane < j) && (mine == cand);
      ok = (cand != forbid) && (__ballot(clash) == 0ull);
    }
    // at most `range` steps: the host has checked that enough ids are free
    for (uint32_t step = 0; step < range && !ok; ++step) {
      uint32_t local = cand - base;
      local = (local + 1 == range) ? 0 : local + 1;
      cand = local + base;
      bool clash = (lane < j) && (mine == cand);
      ok = (cand != forbid) && (__ballot(clash) == 0ull);
    }
    if (lane == j) mine = cand;
  }
  return mine;
}

}  // namespace gnnd
