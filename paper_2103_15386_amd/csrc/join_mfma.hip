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
#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kMB = 256;  // 4 waves = 4 nodes per workgroup
constexpr int32_t kFar = 1 << 24;  // "norm" of an absent row: above every real distance

// Convert float32 rows holding integers 0..255 (or uint8 rows) to int8 rows
// (value - 128) of `dpad` bytes, zero padded, and store the squared norm of
// the shifted row.  `bad` is raised when a float is not such an integer.
template <typename T>
__global__ __launch_bounds__(256) void k_pack_i8(const void* vec_a, const void* vec_b,
                                                 int64_t split, int64_t n, int d, int dpad,
                                                 int8_t* shadow, int32_t* norms, int* bad) {
  const int lane = lane_id();
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
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
  if (lane == 0) norms[row] = acc;
  if (__ballot(is_bad) != 0ull && lane == 0) atomicOr(bad, 1);
}

// min over the 16 accumulator registers of a tile, per lane (= per column), of
// the signed key (row_norm - 2 G) << 6 | row position, rows flagged in `excl`
// skipped.  Row of register r for this lane: 8*(r/4) + 4*half + (r%4).  Adding
// the column's own norm to key >> 6 afterwards gives the squared distance; the
// shift keeps the order because |row_norm - 2 G| stays below 2^25.
constexpr int32_t kNone = 0x7fffffff;

template <bool MASKED>
__device__ inline int32_t tile_col_min(const v16i& g, const int32_t* row_norm_lds, int half,
                                       int row_base, uint32_t excl) {
  int32_t best = kNone;
  const uint32_t ex = excl >> (4 * half);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int4 nr = *reinterpret_cast<const int4*>(row_norm_lds + 8 * q + 4 * half);
    const int32_t nrm[4] = {nr.x, nr.y, nr.z, nr.w};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int r = 4 * q + t;
      const int32_t part = nrm[t] - 2 * g[r];
      int32_t key = (int32_t)(((uint32_t)part << 6) | (uint32_t)(row_base + 8 * q + 4 * half + t));
      if (MASKED) {
        const uint32_t bit = 1u << (8 * q + t);
        key = (ex & bit) ? kNone : key;
      }
      best = key < best ? key : best;
    }
  }
  return best;
}

__device__ inline int32_t both_halves_min(int32_t x) {
  auto sw = __builtin_amdgcn_permlane32_swap((uint32_t)x, (uint32_t)x, false, false);
  int32_t a = (int32_t)sw[0], b = (int32_t)sw[1];
  return a < b ? a : b;
}

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
template <int KSTEPS, bool FCODE, bool MERGE>
__global__ __launch_bounds__(kMB) void k_join_mfma(
    const int8_t* __restrict__ shadow, const int32_t* __restrict__ norms, int dpad, int64_t n,
    int p, int64_t split, const int32_t* __restrict__ snew, const int32_t* __restrict__ sold,
    const int32_t* __restrict__ cnew, const int32_t* __restrict__ cold,
    const uint32_t* __restrict__ kth, uint32_t* pcnt, const uint64_t* __restrict__ poff,
    uint64_t* __restrict__ bins, uint64_t* counters) {
  // per wave: norms of the 128 rows (NEW 0..63, OLD 64..127) and their ids
  __shared__ __attribute__((aligned(16))) int32_t s_norm[4][128];
  __shared__ int32_t s_id[4][128];
  const int wave = threadIdx.x >> 6, lane = lane_id(), half = lane >> 5, col = lane & 31;
  const int64_t s = (int64_t)blockIdx.x * 4 + wave;
  if (s >= n) return;
  const int L = 2 * p;
  const int nn = cnew[s], no = cold[s];
  const bool do_nn = !MERGE && nn > 1;
  if (nn == 0 || (!do_nn && no == 0)) return;
  const int32_t id_new = lane < nn ? snew[s * L + lane] : -1;
  const int32_t id_old = lane < no ? sold[s * L + lane] : -1;

  // operands: block b of a list = its rows 32b..32b+31; lane (col, half) holds
  // bytes [32s + 16 half, +16) of row `col` of the block for every step s
  const int32_t rid_n0 = __shfl(id_new, col, kWave), rid_n1 = __shfl(id_new, 32 + col, kWave);
  const int32_t rid_o0 = __shfl(id_old, col, kWave), rid_o1 = __shfl(id_old, 32 + col, kWave);
  const Operand N0 = load_block<KSTEPS>(shadow, dpad, rid_n0, half);
  const Operand N1 = load_block<KSTEPS>(shadow, dpad, nn > 32 ? rid_n1 : -1, half);
  const Operand O0 = load_block<KSTEPS>(shadow, dpad, rid_o0, half);
  const Operand O1 = load_block<KSTEPS>(shadow, dpad, no > 32 ? rid_o1 : -1, half);

  const int32_t nrm_new = id_new >= 0 ? norms[id_new] : kFar;
  const int32_t nrm_old = id_old >= 0 ? norms[id_old] : kFar;
  s_norm[wave][lane] = nrm_new;
  s_norm[wave][64 + lane] = nrm_old;
  s_id[wave][lane] = id_new;
  s_id[wave][64 + lane] = id_old;
  // the wave reads these back below: order its own LDS writes before its reads
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // objects sampled both as NEW and as OLD: that pair is not a pair.  eq_old =
  // position in the OLD list of this lane's NEW object (or -1), and vice versa.
  int eq_old = -1, eq_new = -1;
  uint32_t dups = 0;
  if (no > 0) {
    for (int i = 0; i < no; ++i) {
      const int32_t oid = __builtin_amdgcn_readlane(id_old, i);
      if (id_new == oid) eq_old = i;
    }
    const uint64_t m = __ballot(eq_old >= 0);
    dups = (uint32_t)__popcll(m);
    if (dups) {
      for (int i = 0; i < nn; ++i) {
        const int32_t nid = __builtin_amdgcn_readlane(id_new, i);
        if (id_old == nid && id_old >= 0) eq_new = i;
      }
    }
  }
  // per-lane exclusion masks (bit r = row r of the block is not a partner of
  // this lane's column object); lanes l and l+32 serve column l%32 of block 0,
  // results of block 1 are selected into lanes 32..63 at the end
  const int eq_old_c0 = __shfl(eq_old, col, kWave), eq_old_c1 = __shfl(eq_old, 32 + col, kWave);
  const int eq_new_c0 = __shfl(eq_new, col, kWave), eq_new_c1 = __shfl(eq_new, 32 + col, kWave);
  // merge mode: rows whose set equals the column object's set are excluded
  uint32_t cls_new0 = 0, cls_new1 = 0, cls_old0 = 0, cls_old1 = 0;
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
  int32_t a0 = kNone, a1 = kNone;  // NEW column blocks: nearest other NEW
  int32_t b0 = kNone, b1 = kNone;  // NEW column blocks: nearest OLD
  int32_t c0 = kNone, c1 = kNone;  // OLD column blocks: nearest NEW

  if (do_nn) {
    {  // rows N0, columns N0: the diagonal pairs an object with itself
      v16i g = gram<KSTEPS>(N0, N0);
      a0 = min(a0, tile_col_min<true>(g, normN, half, 0, 1u << col));
    }
    if (nn > 32) {
      {
        v16i g = gram<KSTEPS>(N1, N0);
        a0 = min(a0, tile_col_min<false>(g, normN + 32, half, 32, 0u));
      }
      {
        v16i g = gram<KSTEPS>(N0, N1);
        a1 = min(a1, tile_col_min<false>(g, normN, half, 0, 0u));
      }
      {
        v16i g = gram<KSTEPS>(N1, N1);
        a1 = min(a1, tile_col_min<true>(g, normN + 32, half, 32, 1u << col));
      }
    }
  }
  if (no > 0) {
    // columns = NEW objects, rows = OLD objects: nearest OLD of every NEW
    {
      v16i g = gram<KSTEPS>(O0, N0);
      b0 = min(b0, masked_no ? tile_col_min<true>(g, normO, half, 0,
                                                  excl_rows(eq_old_c0, 0, cls_old0, rid_n0))
                             : tile_col_min<false>(g, normO, half, 0, 0u));
    }
    if (no > 32) {
      v16i g = gram<KSTEPS>(O1, N0);
      b0 = min(b0, masked_no ? tile_col_min<true>(g, normO + 32, half, 32,
                                                  excl_rows(eq_old_c0, 1, cls_old1, rid_n0))
                             : tile_col_min<false>(g, normO + 32, half, 32, 0u));
    }
    if (nn > 32) {
      {
        v16i g = gram<KSTEPS>(O0, N1);
        b1 = min(b1, masked_no ? tile_col_min<true>(g, normO, half, 0,
                                                    excl_rows(eq_old_c1, 0, cls_old0, rid_n1))
                               : tile_col_min<false>(g, normO, half, 0, 0u));
      }
      if (no > 32) {
        v16i g = gram<KSTEPS>(O1, N1);
        b1 = min(b1, masked_no ? tile_col_min<true>(g, normO + 32, half, 32,
                                                    excl_rows(eq_old_c1, 1, cls_old1, rid_n1))
                               : tile_col_min<false>(g, normO + 32, half, 32, 0u));
      }
    }
    // columns = OLD objects, rows = NEW objects: nearest NEW of every OLD
    {
      v16i g = gram<KSTEPS>(N0, O0);
      c0 = min(c0, masked_no ? tile_col_min<true>(g, normN, half, 0,
                                                  excl_rows(eq_new_c0, 0, cls_new0, rid_o0))
                             : tile_col_min<false>(g, normN, half, 0, 0u));
    }
    if (nn > 32) {
      v16i g = gram<KSTEPS>(N1, O0);
      c0 = min(c0, masked_no ? tile_col_min<true>(g, normN + 32, half, 32,
                                                  excl_rows(eq_new_c0, 1, cls_new1, rid_o0))
                             : tile_col_min<false>(g, normN + 32, half, 32, 0u));
    }
    if (no > 32) {
      {
        v16i g = gram<KSTEPS>(N0, O1);
        c1 = min(c1, masked_no ? tile_col_min<true>(g, normN, half, 0,
                                                    excl_rows(eq_new_c1, 0, cls_new0, rid_o1))
                               : tile_col_min<false>(g, normN, half, 0, 0u));
      }
      if (nn > 32) {
        v16i g = gram<KSTEPS>(N1, O1);
        c1 = min(c1, masked_no ? tile_col_min<true>(g, normN + 32, half, 32,
                                                    excl_rows(eq_new_c1, 1, cls_new1, rid_o1))
                               : tile_col_min<false>(g, normN + 32, half, 32, 0u));
      }
    }
  }
  // combine the two row halves; lanes 0..31 take column block 0, lanes 32..63 block 1
  a0 = both_halves_min(a0); a1 = both_halves_min(a1);
  b0 = both_halves_min(b0); b1 = both_halves_min(b1);
  c0 = both_halves_min(c0); c1 = both_halves_min(c1);
  const int32_t ra = half ? a1 : a0, rb = half ? b1 : b0, rc = half ? c1 : c0;

  // lane l now answers for sample l of its list, three results
  uint32_t found_total = 0, over_total = 0;
#pragma unroll
  for (int kind = 0; kind < 3; ++kind) {
    const int32_t res = kind == 0 ? ra : (kind == 1 ? rb : rc);
    const int32_t self = kind == 2 ? id_old : id_new;
    const int32_t self_norm = kind == 2 ? nrm_old : nrm_new;
    const int32_t part = res >> 6;  // row_norm - 2 G (arithmetic shift); absent rows sit at kFar
    const bool found = self >= 0 && res != kNone && part < (kFar >> 1);
    const int32_t dist = part + self_norm;
    const int pos = res & 63;
    const int32_t other = found ? s_id[wave][(kind == 0 ? 0 : (kind == 1 ? 64 : 0)) + pos] : 0;
    const uint32_t code = FCODE ? ord_f32((float)dist) : ord_i32(dist);
    const bool pass = found && code <= kth[found ? self : 0];
    bool overflow = false;
    if (pass) {  // into the destination's segment of the proposal array
      const uint64_t beg = poff[self], cap = poff[self + 1] - beg;
      const uint32_t pos = atomicAdd(&pcnt[self], 1u);
      if (pos < cap) bins[beg + pos] = make_entry(code, (uint32_t)other, 3u);
      else overflow = true;
    }
    found_total += (uint32_t)__popcll(__ballot(found));
    over_total += (uint32_t)__popcll(__ballot(overflow));
  }
  if (lane == 0) {
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
    if (found_total) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_PROPS),
                               (unsigned long long)found_total);
    if (over_total) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_OVERFLOW),
                              (unsigned long long)over_total);
    if (ev) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_EVALS), (unsigned long long)ev);
  }
}

template <int KSTEPS>
static void launch_k(bool fcode, bool merge, unsigned grid, hipStream_t st, const int8_t* shadow,
                     const int32_t* norms, int dpad, const Shape& sh, const DevState& ds) {
#define GNND_ARGS shadow, norms, dpad, sh.n, sh.p, sh.split, ds.snew, ds.sold, ds.cnew, ds.cold, \
                  ds.kth, ds.pcnt, ds.poff, ds.bins, ds.counters
  if (fcode) {
    if (merge) k_join_mfma<KSTEPS, true, true><<<grid, kMB, 0, st>>>(GNND_ARGS);
    else k_join_mfma<KSTEPS, true, false><<<grid, kMB, 0, st>>>(GNND_ARGS);
  } else {
    if (merge) k_join_mfma<KSTEPS, false, true><<<grid, kMB, 0, st>>>(GNND_ARGS);
    else k_join_mfma<KSTEPS, false, false><<<grid, kMB, 0, st>>>(GNND_ARGS);
  }
#undef GNND_ARGS
}

hipError_t launch_join_mfma(const Shape& sh, const DevState& ds, bool merge_mode,
                            hipStream_t st) {
  const int dpad = (sh.d + 31) & ~31;
  const int ksteps = dpad / 32;
  const unsigned grid = (unsigned)((sh.n + 3) / 4);
  const bool fcode = sh.metric != kL2U8;
  switch (ksteps) {
    case 1: launch_k<1>(fcode, merge_mode, grid, st, ds.shadow, ds.norms, dpad, sh, ds); break;
    case 2: launch_k<2>(fcode, merge_mode, grid, st, ds.shadow, ds.norms, dpad, sh, ds); break;
    case 3: launch_k<3>(fcode, merge_mode, grid, st, ds.shadow, ds.norms, dpad, sh, ds); break;
    default: launch_k<4>(fcode, merge_mode, grid, st, ds.shadow, ds.norms, dpad, sh, ds);
  }
  return hipGetLastError();
}

hipError_t launch_pack_i8(const Shape& sh, const DevState& ds, int* bad_flag_dev,
                          hipStream_t st) {
  const int dpad = (sh.d + 31) & ~31;
  const unsigned grid = (unsigned)((sh.n + 3) / 4);
  if (sh.metric == kL2U8)
    k_pack_i8<uint8_t><<<grid, 256, 0, st>>>(sh.vec_a, sh.vec_b, sh.split, sh.n, sh.d, dpad,
                                             ds.shadow, ds.norms, bad_flag_dev);
  else
    k_pack_i8<float><<<grid, 256, 0, st>>>(sh.vec_a, sh.vec_b, sh.split, sh.n, sh.d, dpad,
                                           ds.shadow, ds.norms, bad_flag_dev);
  return hipGetLastError();
}

}  // namespace gnnd
