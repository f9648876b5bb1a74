// Cross-matching (Sec. 4.2) and selective nearest-object search (Sec. 4.3,
// Alg. 2) for float32 vectors, inner products on the matrix cores (Sec. 4.2
// treats NEW x OLD as a tiled matrix product), results exactly those of the
// per-pair evaluation in dimension order.
//
// One wavefront per node at a time, no barriers between wavefronts, four steps:
//  1. The inner products of the block [NEW x (NEW | OLD)] of the node's <= 64 NEW
//     and <= 64 OLD sample vectors are accumulated by v_mfma_f32_16x16x4_f32 in
//     16 x 16 blocks, all of them in registers; only blocks that hold list
//     entries are computed (lower block triangle of NEW x NEW).  The operands
//     come straight from memory: four lanes read 64 consecutive bytes of a row,
//     which is the matrix instruction's own operand layout, 16 dimensions per
//     step, two steps (both halves of a 128-byte line) requested together.
//  2. Inner product and squared norms give every pair an approximate distance
//     whose difference from the canonical sum (one fused multiply-add per
//     dimension, in dimension order) is bounded by eps(pair), see pair_bounds.
//  3. Per sample and direction (NEW towards NEW, NEW towards OLD, OLD towards
//     NEW) the partners that may still be its nearest one are kept:
//     approx - eps <= min over partners of (approx + eps), found by reductions
//     over the accumulator blocks.  Partners whose lower bound already lies
//     beyond the threshold of the sample's list are dropped, for nothing at that
//     distance is handed on.  One partner is left as a rule, seldom a few, often
//     none.
//  4. The vectors concerned are read once more, the same way, and pass through
//     an LDS tile 16 dimensions at a time, where one lane per sample accumulates
//     the canonical distances of the partners left; the smallest (distance, id)
//     is the result.
// The nodes are listed by the number of blocks of 16 samples they fill
// (k_gram_classify), and each class has its own build of the kernel, with the
// registers and the LDS tile that its blocks need, run by persistent wavefronts
// over the class's list.
#include <stddef.h>

#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

namespace {

constexpr int kWC = 16;    // dimensions per step of the inner-product loop
constexpr int kWLD = kWC + 4;  // row stride (floats) of the LDS tile of step 4: 16-byte aligned
                               // rows, and the 64 lanes of a 16-byte access spread evenly
                               // over the banks
constexpr int kWCand = 2;  // canonical sums per lane and direction in one pass over the vectors

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Everything one wavefront (= one workgroup) keeps in LDS.  Rows 0..63 are the NEW samples,
// rows 64..127 the OLD samples; slots 0..63 stand for "NEW sample towards NEW", 64..127 for
// "NEW sample towards OLD", 128..191 for "OLD sample towards NEW".
struct GramLds {
  int32_t ids[128];
  float norms[128];   // squared norms
  // what the approximate distance needs of a sample: its squared norm (cosine: one over its
  // norm, 0 for a zero vector); NaN for the empty rows of a 16-row block, which makes every
  // bound of their pairs NaN: never a minimum, never below a limit
  float weight[128];
  uint32_t kth[128];   // threshold of each sample's list
  uint32_t upper[192];  // smallest upper bound of a partner's distance (order-preserving code)
  float limit[192];     // what a partner's lower bound must not exceed
  unsigned long long cmask[192];  // the partners left (bit per partner)
};

// The builds of the kernel: build c holds up to rbm blocks of 16 NEW and com blocks of 16 OLD
// samples and is compiled for `waves` wavefronts per SIMD.  The shapes follow what a
// construction meets: every node of the first iteration has NEW samples only; in the next few
// iterations most have 33 to 48 NEW samples and up to 16 OLD ones; later the NEW samples dwindle
// and the OLD ones fill up.
struct GramShape {
  int rbm, com, waves;
};
__host__ __device__ constexpr GramShape gram_shape(int cls) {
  return cls == 0   ? GramShape{4, 0, 4}
         : cls == 1 ? GramShape{1, 2, 4}
         : cls == 2 ? GramShape{3, 1, 4}
         : cls == 3 ? GramShape{1, 4, 4}
         : cls == 4 ? GramShape{2, 4, 3}
         : cls == 5 ? GramShape{4, 2, 3}
                    : GramShape{4, 4, 2};
}
// Which build takes a node with rb blocks of NEW and co blocks of OLD samples: the cheapest
// one that holds them.
__host__ __device__ constexpr int gram_class(int rb, int co) {
  return co == 0 ? 0 : (rb <= 1 && co <= 2) ? 1 : (rb <= 3 && co <= 1) ? 2 : rb <= 1 ? 3
         : rb <= 2 ? 4 : co <= 2 ? 5 : 6;
}
static_assert(kGramClasses == 7, "gram_shape and gram_class list seven builds");
// first LDS row of operand block q of a build with RBM blocks of NEW samples
template <int RBM>
__device__ constexpr int block_row(int q) {
  return q < RBM ? 16 * q : 64 + 16 * (q - RBM);
}

// What a wavefront has counted over its nodes (the same in every lane).
struct GramTally {
  uint64_t found = 0, passed = 0, overflow = 0, evals = 0;
};

template <int METRIC, bool WHOLE, int RBM, int COM>
__device__ __forceinline__ void gram_node(GramLds& S, float* tile, const VecSrc& vs, int64_t s,
                                          int p, int merge_mode,
                                          const int32_t* __restrict__ snew,
                                          const int32_t* __restrict__ sold, int nn, int no,
                                          const NodeMeta* __restrict__ meta, uint64_t* pslot,
                                          uint64_t slots, uint64_t* __restrict__ bins,
                                          GramTally& tally) {
  using TR = JoinTraits<METRIC>;
  constexpr int NB = RBM + COM;  // operand blocks: NEW blocks first, then OLD blocks
  auto tile_row = [](int row) { return row < 64 ? row : row - 64 + 16 * RBM; };
  constexpr uint32_t kNone = 0xffffffffu;
  const float kInf = __uint_as_float(0x7f800000u), kNaN = __uint_as_float(0x7fc00000u);
  // (taken anew for every node: what depends on the lane is worked out again per node
  // instead of being held in registers across the loop over nodes)
  int lane = threadIdx.x;
  asm volatile("" : "+v"(lane));
  const int L = 2 * p;
  const int64_t split = vs.split;
  const int d = vs.d;
  const float* const set_a = reinterpret_cast<const float*>(vs.a);
  const float* const set_b = reinterpret_cast<const float*>(vs.b);
  auto row_of = [=](int32_t id) {
    return (int64_t)id < split ? set_a + (int64_t)id * d : set_b + ((int64_t)id - split) * d;
  };
  const bool do_nn = !merge_mode && nn > 1;
  // lane l holds NEW sample l and OLD sample l
  const int32_t idn = lane < nn ? snew[s * L + lane] : -1;
  const int32_t ido = lane < no ? sold[s * L + lane] : -1;
  S.ids[lane] = idn;
  S.ids[64 + lane] = ido;
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    S.upper[64 * t + lane] = kNone;
    S.cmask[64 * t + lane] = 0ull;
  }
  __syncthreads();

  const int RB = (nn + 15) >> 4;  // 16-row blocks of NEW samples
  const int CO = (no + 15) >> 4;  // 16-column blocks of OLD samples
  const bool aligned = (d & 3) == 0;
  const int l16 = lane & 15, g4 = (lane >> 4) * 4;
  // Lane (l16, g) holds dimensions 4 g .. 4 g + 3 (of the 16 of a step) of row l16 of a block,
  // for either operand: which dimension goes to which step of the contraction does not matter
  // as long as both operands agree.  rows[q] / rows[4 + q]: this lane's row of NEW / OLD block
  // q.  An empty list place reads the node's first NEW sample instead: whatever stands in its
  // row or column of a block, the NaN weight of the place keeps it out of every result.
  const float* rows[NB];
  {
    const float* any_row = row_of(S.ids[0]) + g4;
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      const int32_t id = S.ids[block_row<RBM>(q) + l16];
      rows[q] = id >= 0 ? row_of(id) + g4 : any_row;
    }
  }
  // The operands of two steps, 32 dimensions of every row, are requested together: the two
  // 64-byte pieces of a row are the halves of one 128-byte line where rows are aligned to
  // lines, and memory serves a line requested at once faster than its halves requested one
  // after the other (measured on random rows: 6.5 against 5.5 TB/s).  Always all 2 NB loads,
  // so that the number of loads in flight is known where the products wait for them; where
  // the vector ends after the first of the two steps, the second reads that step once more.
  const int d_last = ((d - 1) / kWC) * kWC;
  auto fetch_one = [&](const float* src, int j) {
    if (WHOLE) return *reinterpret_cast<const float4*>(src);
    // dimensions beyond the last one count as zeros
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (aligned && j + 3 < d) {
      v = *reinterpret_cast<const float4*>(src);
    } else {
      if (j + 0 < d) v.x = src[0];
      if (j + 1 < d) v.y = src[1];
      if (j + 2 < d) v.z = src[2];
      if (j + 3 < d) v.w = src[3];
    }
    return v;
  };
  auto fetch2 = [&](float4* fa, float4* fb, int d0) {
    const int d1 = d0 + kWC < d_last ? d0 + kWC : d_last;
#pragma unroll
    for (int q = 0; q < NB; ++q) {
      fa[q] = fetch_one(rows[q] + d0, d0 + g4);
      fb[q] = fetch_one(rows[q] + d1, d1 + g4);
    }
  };
  float4 opa[NB], opb[NB];
  fetch2(opa, opb, 0);

  {
    // one 8-byte record per sample: the threshold of its list and its squared norm
    // (launch_gram_norms put the float's bits where the int8 join keeps its integer norm)
    const uint2 mn = idn >= 0 ? *reinterpret_cast<const uint2*>(&meta[idn]) : make_uint2(0u, 0u);
    const uint2 mo = ido >= 0 ? *reinterpret_cast<const uint2*>(&meta[ido]) : make_uint2(0u, 0u);
    const uint32_t kthn = mn.x, ktho = mo.x;
    const float nrmn = __uint_as_float(mn.y), nrmo = __uint_as_float(mo.y);
    auto weight_of = [&](int32_t id, float nrm) {
      float w = nrm;
      if (METRIC == kCosineF32) w = nrm > 0.f ? 1.0f / sqrtf(nrm) : 0.f;
      return id >= 0 ? w : kNaN;
    };
    S.norms[lane] = nrmn;
    S.norms[64 + lane] = nrmo;
    S.kth[lane] = kthn;
    S.kth[64 + lane] = ktho;
    S.weight[lane] = weight_of(idn, nrmn);
    S.weight[64 + lane] = weight_of(ido, nrmo);
  }
  // An object sampled as NEW and as OLD here is no pair (sample lists are ascending in id:
  // binary search); a merge only joins objects of different sets.
  uint32_t n_dup, new_first, old_first;
  {
    int lo = 0, hi = nn;
    while (__ballot(lo < hi) != 0ull) {
      if (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (S.ids[mid] < ido) lo = mid + 1;
        else hi = mid;
      }
    }
    n_dup = (uint32_t)__popcll(__ballot(ido >= 0 && lo < nn && S.ids[lo] == ido));
    new_first = (uint32_t)__popcll(__ballot(idn >= 0 && (int64_t)idn < split));
    old_first = (uint32_t)__popcll(__ballot(ido >= 0 && (int64_t)ido < split));
  }

  // ---- 1. inner products --------------------------------------------------------------
  // acc_no[rb][cb]: NEW rows 16 rb.. x OLD rows 16 cb..; acc_nn[rb (rb + 1) / 2 + cb], cb <= rb:
  // NEW rows 16 rb.. x NEW rows 16 cb..
  f32x4 acc_no[RBM][COM > 0 ? COM : 1], acc_nn[RBM * (RBM + 1) / 2];
#pragma unroll
  for (int rb = 0; rb < RBM; ++rb)
#pragma unroll
    for (int cb = 0; cb < COM; ++cb) acc_no[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < RBM * (RBM + 1) / 2; ++t) acc_nn[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto mfma4 = [](f32x4& acc, const float4& a, const float4& b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, acc, 0, 0, 0);
  };
  auto products = [&](const float4* op) {
#pragma unroll
    for (int rb = 0; rb < RBM; ++rb) {
      if (rb < RB) {  // uniform
#pragma unroll
        for (int cb = 0; cb < COM; ++cb)
          if (cb < CO) mfma4(acc_no[rb][cb], op[rb], op[RBM + cb]);
        if (do_nn) {
#pragma unroll
          for (int cb = 0; cb <= rb; ++cb) mfma4(acc_nn[rb * (rb + 1) / 2 + cb], op[rb], op[cb]);
        }
      }
    }
  };
  // steps 0, 2, 4, ... use opa, steps 1, 3, ... opb
  for (int d0 = 0;;) {
    products(opa);
    if (d0 + kWC < d) products(opb);
    d0 += 2 * kWC;
    if (d0 >= d) break;
    fetch2(opa, opb, d0);
  }

  // ---- 2. + 3. partners that may be the nearest one --------------------------------------
  // Bound eps of |approximate distance - canonical distance| (u = 2^-24, c0 = (6 d + 16) u):
  // an inner product of d terms accumulated in float32 in any order and with any rounding of
  // the partial sums is within 2 d u sum|a_i b_i| of the true one, the canonical sums within
  // (d + 2) u of theirs, the norms within d u; sum|a_i b_i| <= sqrt(na nb) <= (na + nb) / 2.
  // Squared L2, na + nb - 2 dot: the errors of na, nb, 2 dot and of the sum of differences
  // add up to less than (5 d + 14) u (na + nb); c0 (na + nb) is used.  1 - dot: half of that
  // plus the rounding of the subtraction (2^-22 covers both sides).  Cosine,
  // 1 - dot / sqrt(na nb): the same relative to the denominator, plus the roundings of the
  // reciprocal root and the products.
  const float c0 = (float)(6 * d + 16) * 5.9604645e-8f;
  const bool with_dups = !merge_mode && n_dup != 0;
  // Pair (row R = arow + 4 g + r, column brow + l16) of a block: lane (l16, g) of the block's
  // accumulator holds rows 4 g .. 4 g + 3 of column l16.
  auto pair_bounds = [&](float dot, int arow, int brow, int r, float wc, int32_t idc, float& val,
                         float& e) {
    const int R = arow + g4 + r;
    const float wr = S.weight[R];
    if (METRIC == kCosineF32) {
      val = 1.0f - dot * wr * wc;
      e = c0 + 4.7683716e-7f;
    } else {
      const float t = wr + wc;
      val = METRIC == kL2F32 ? t - 2.0f * dot : 1.0f - dot;
      e = METRIC == kL2F32 ? c0 * t : c0 * t + 2.3841858e-7f;
    }
    if (brow == arow) {  // diagonal block of NEW x NEW: strict lower triangle, every pair once
      if (l16 >= g4 + r) val = kNaN;
    } else if (brow >= 64 && (with_dups || merge_mode)) {
      const int32_t idr = S.ids[R];
      if (merge_mode ? (((int64_t)idr < split) == ((int64_t)idc < split)) : idr == idc) val = kNaN;
    }
  };
  // A pair of a NEW x OLD block serves the NEW sample's search among the OLD ones and the OLD
  // sample's among the NEW ones, a pair of a NEW x NEW block both of its samples.  First the
  // smallest upper bound per sample and direction: along the rows through the 16 lanes of a
  // lane row, along the columns inside the lane and over the four lane rows, then through LDS.
  auto fold_upper = [&](const f32x4& acc, int arow, int brow) {
    const bool nn_block = brow < 64;
    const int col = brow + l16;
    const float wc = S.weight[col];
    const int32_t idc = S.ids[col];
    float col_min = kInf;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float val, e;
      pair_bounds(acc[r], arow, brow, r, wc, idc, val, e);
      float row_min = fminf(val + e, kInf);
      col_min = fminf(col_min, row_min);
#pragma unroll
      for (int j = 1; j < 16; j <<= 1)
        row_min = fminf(row_min, __uint_as_float(xor_lanes(__float_as_uint(row_min), j, lane)));
      if (l16 == 0 && row_min < kInf)
        atomicMin(&S.upper[(nn_block ? 0 : 64) + arow + g4 + r], ord_f32(row_min));
    }
    col_min = fminf(col_min, __uint_as_float(xor_lanes(__float_as_uint(col_min), 16, lane)));
    col_min = fminf(col_min, __uint_as_float(xor_lanes(__float_as_uint(col_min), 32, lane)));
    if (g4 == 0 && col_min < kInf) atomicMin(&S.upper[nn_block ? col : 64 + col], ord_f32(col_min));
  };
  // Then every pair whose lower bound exceeds neither that nor the threshold of the sample's
  // list is entered in the sample's set of partners.
  auto fold_partners = [&](const f32x4& acc, int arow, int brow) {
    const bool nn_block = brow < 64;
    const int col = brow + l16;
    const float wc = S.weight[col];
    const int32_t idc = S.ids[col];
    const int col_slot = nn_block ? col : 64 + col;
    const float col_limit = S.limit[col_slot];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float val, e;
      pair_bounds(acc[r], arow, brow, r, wc, idc, val, e);
      const float lower = val - e;
      const int R = arow + g4 + r;
      const int row_slot = (nn_block ? 0 : 64) + R;
      if (lower <= S.limit[row_slot]) atomicOr(&S.cmask[row_slot], 1ull << (col & 63));
      if (lower <= col_limit) atomicOr(&S.cmask[col_slot], 1ull << R);
    }
  };
  auto over_blocks = [&](auto fold) {
#pragma unroll
    for (int rb = 0; rb < RBM; ++rb) {
      if (rb < RB) {  // uniform
#pragma unroll
        for (int cb = 0; cb < COM; ++cb)
          if (cb < CO) fold(acc_no[rb][cb], 16 * rb, 64 + 16 * cb);
        if (do_nn) {
#pragma unroll
          for (int cb = 0; cb <= rb; ++cb) fold(acc_nn[rb * (rb + 1) / 2 + cb], 16 * rb, 16 * cb);
        }
      }
    }
  };
  over_blocks(fold_upper);
  __syncthreads();
#pragma unroll
  for (int t = 0; t < 3; ++t)
    S.limit[64 * t + lane] = unord_f32(vmin(S.upper[64 * t + lane], S.kth[t == 2 ? 64 + lane : lane]));
  __syncthreads();
  over_blocks(fold_partners);
  __syncthreads();

  // ---- 4. canonical distances of the partners left --------------------------------------
  // direction 0: NEW sample `lane` towards NEW, 1: NEW sample towards OLD, 2: OLD sample
  // towards NEW
  uint64_t cand[3], best[3];
  bool found[3];
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    const bool searching = (t == 2 ? ido : idn) >= 0 && (t != 0 || do_nn);
    found[t] = searching && S.upper[64 * t + lane] != kNone;
    cand[t] = searching ? S.cmask[64 * t + lane] : 0ull;
    best[t] = kKeyMax;
  }
  // The vectors concerned come the same way as in step 1 (two steps in flight, the others'
  // places read the node's first NEW sample) and are laid out in LDS row by row, 16
  // dimensions at a time; lane l then adds these 16 dimensions, in order, to the sums of its
  // pairs.
  while (__ballot((cand[0] | cand[1] | cand[2]) != 0ull) != 0ull) {
    int crow[3][kWCand], c[3];
    bool lanes_with[3][kWCand];  // some lane holds a partner number i in direction t
    unsigned long long m0 = 0ull, m1 = 0ull;  // rows this lane reads: NEW rows, OLD rows
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      c[t] = 0;
#pragma unroll
      for (int i = 0; i < kWCand; ++i) {
        crow[t][i] = 0;
        if (cand[t] != 0ull) {
          const int v = __ffsll((unsigned long long)cand[t]) - 1;
          cand[t] &= cand[t] - 1;
          crow[t][i] = t == 1 ? 64 + v : v;
          (t == 1 ? m1 : m0) |= 1ull << v;
          c[t] = i + 1;
        }
        lanes_with[t][i] = __ballot(c[t] > i) != 0ull;
      }
      if (c[t] > 0) (t == 2 ? m1 : m0) |= 1ull << lane;
    }
    // all lanes' rows: OR over the wavefront
#pragma unroll
    for (int j = 1; j < 64; j <<= 1) {
      m0 |= xor_lanes((uint64_t)m0, j, lane);
      m1 |= xor_lanes((uint64_t)m1, j, lane);
    }
    {
      const float* any_row = row_of(S.ids[0]) + g4;
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        const int row = block_row<RBM>(q) + l16;
        const int32_t id = S.ids[row];
        const bool wanted = (((row < 64 ? m0 : m1) >> (row & 63)) & 1ull) != 0;  // then id >= 0
        rows[q] = wanted ? row_of(id) + g4 : any_row;
      }
    }
    float sum[3][kWCand];
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int i = 0; i < kWCand; ++i) sum[t][i] = 0.f;
    auto sums = [&](const float4* op, int d0) {
      __syncthreads();  // the tile has been read
#pragma unroll
      for (int q = 0; q < NB; ++q)
        *reinterpret_cast<float4*>(tile + (16 * q + l16) * kWLD + g4) = op[q];
      __syncthreads();
      const int width = (d - d0) < kWC ? (d - d0) : kWC;
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        if (lanes_with[t][0]) {  // uniform
          const float* pa = tile + tile_row(t == 2 ? 64 + lane : lane) * kWLD;
          int j = 0;
          for (; j + 3 < width; j += 4) {
            const float4 va = *reinterpret_cast<const float4*>(pa + j);
#pragma unroll
            for (int i = 0; i < kWCand; ++i) {
              if (lanes_with[t][i]) {
                const float4 vb =
                    *reinterpret_cast<const float4*>(tile + tile_row(crow[t][i]) * kWLD + j);
                TR::step(va.x, vb.x, sum[t][i]);
                TR::step(va.y, vb.y, sum[t][i]);
                TR::step(va.z, vb.z, sum[t][i]);
                TR::step(va.w, vb.w, sum[t][i]);
              }
            }
          }
          for (; j < width; ++j) {
#pragma unroll
            for (int i = 0; i < kWCand; ++i)
              if (lanes_with[t][i]) TR::step(pa[j], tile[tile_row(crow[t][i]) * kWLD + j], sum[t][i]);
          }
        }
      }
    };
    fetch2(opa, opb, 0);
    for (int d0 = 0;;) {
      sums(opa, d0);
      if (d0 + kWC < d) sums(opb, d0 + kWC);
      d0 += 2 * kWC;
      if (d0 >= d) break;
      fetch2(opa, opb, d0);
    }
#pragma unroll
    for (int t = 0; t < 3; ++t) {
#pragma unroll
      for (int i = 0; i < kWCand; ++i) {
        if (i < c[t]) {
          const uint64_t code =
              (uint64_t)TR::code(sum[t][i], S.norms[t == 2 ? 64 + lane : lane], S.norms[crow[t][i]]) << 32;
          best[t] = vmin(best[t], code | (uint32_t)S.ids[crow[t][i]]);
        }
      }
    }
  }

  // ---- hand the results on --------------------------------------------------------------
  uint32_t n_found = 0, n_pass = 0, n_over = 0;
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    const int32_t self = t == 2 ? ido : idn;
    const uint32_t kth_self = S.kth[t == 2 ? 64 + lane : lane];
    const bool pass = best[t] != kKeyMax && (uint32_t)(best[t] >> 32) <= kth_self;
    bool over = false;
    if (pass) {
      // one returning add yields the start of the destination's segment of the proposal
      // array and this result's place in it
      const uint64_t w = atomicAdd(reinterpret_cast<unsigned long long*>(&pslot[self]), 1ull);
      const uint64_t at = (w >> kSlotCountBits) + (w & kSlotCountMask);
      if (at < slots) bins[at] = make_entry((uint32_t)(best[t] >> 32), (uint32_t)best[t], 3u);
      else over = true;
    }
    n_found += (uint32_t)__popcll(__ballot(found[t]));
    n_pass += (uint32_t)__popcll(__ballot(pass));
    n_over += (uint32_t)__popcll(__ballot(over));
  }
  tally.found += n_found;
  tally.passed += n_pass;
  tally.overflow += n_over;
  // pairs that count as evaluated: NEW x OLD without the objects sampled as both (a merge:
  // pairs across the two sets), and all pairs of NEW samples
  const uint64_t fa = new_first, fb = old_first;
  tally.evals += merge_mode ? fa * ((uint64_t)no - fb) + ((uint64_t)nn - fa) * fb
                            : (uint64_t)nn * no - n_dup;
  if (do_nn) tally.evals += (uint64_t)nn * (nn - 1) / 2;
}

// The nodes that have something to evaluate, listed by class (list c at nodes + c n, its
// length in count[c]; the order inside a list is of no consequence).  A workgroup takes
// kClassifyNodes consecutive nodes, numbers those of each class in LDS and reserves their
// places with one addition per class.
constexpr int kClassifyPerThread = 16;
constexpr int kClassifyNodes = 256 * kClassifyPerThread;
__global__ __launch_bounds__(256) void k_gram_classify(int64_t n, int merge_mode,
                                                       const int32_t* __restrict__ cnew,
                                                       const int32_t* __restrict__ cold,
                                                       int32_t* nodes, uint32_t* count) {
  __shared__ uint32_t here[kGramClasses], base[kGramClasses];
  const int64_t first = block_linear() * kClassifyNodes;
  if (threadIdx.x < kGramClasses) here[threadIdx.x] = 0u;
  __syncthreads();
  int32_t place[kClassifyPerThread];  // class + kGramClasses x (number within the workgroup)
#pragma unroll
  for (int j = 0; j < kClassifyPerThread; ++j) {
    const int64_t s = first + j * 256 + threadIdx.x;
    place[j] = -1;
    if (s < n) {
      const int nn = cnew[s], no = cold[s];
      const bool do_nn = !merge_mode && nn > 1;
      if (nn != 0 && (do_nn || no != 0)) {
        const int cls = gram_class((nn + 15) >> 4, (no + 15) >> 4);
        place[j] = cls + kGramClasses * (int32_t)atomicAdd(&here[cls], 1u);
      }
    }
  }
  __syncthreads();
  if (threadIdx.x < kGramClasses && here[threadIdx.x] != 0u)
    base[threadIdx.x] = atomicAdd(&count[threadIdx.x], here[threadIdx.x]);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kClassifyPerThread; ++j) {
    if (place[j] >= 0) {
      const int cls = place[j] % kGramClasses;
      nodes[(int64_t)cls * n + base[cls] + place[j] / kGramClasses] =
          (int32_t)(first + j * 256 + threadIdx.x);
    }
  }
}

// WHOLE: the dimension is a multiple of 16, every step reads 16 present dimensions.
// CLS: the build (gram_shape); it takes the nodes of its class from that class's list.  The
// accumulators of all blocks and two sets of operands live in registers, and a build for
// fewer blocks runs more wavefronts per SIMD and reads and multiplies fewer empty blocks.
// Persistent wavefronts: wavefront w takes the list's places w, w + (number of wavefronts), ...
template <int METRIC, bool WHOLE, int CLS>
__global__ __launch_bounds__(kWave)
__attribute__((amdgpu_waves_per_eu(gram_shape(CLS).waves, gram_shape(CLS).waves))) void k_join_gram(
    VecSrc vs, int64_t n, int p, int merge_mode, const int32_t* __restrict__ snew,
    const int32_t* __restrict__ sold, const int32_t* __restrict__ cnew,
    const int32_t* __restrict__ cold, const NodeMeta* __restrict__ meta, uint64_t* pslot,
    uint64_t slots, uint64_t* __restrict__ bins, uint64_t* counters,
    const int32_t* __restrict__ nodes, const uint32_t* __restrict__ count) {
  constexpr int RBM = gram_shape(CLS).rbm, COM = gram_shape(CLS).com;
  constexpr int NB = RBM + COM;
  constexpr int cls = CLS;
  __shared__ __attribute__((aligned(16))) GramLds S;
  // step 4: 16 dimensions of every vector the build can hold, operand block after operand block
  __shared__ __attribute__((aligned(16))) float tile[NB * 16 * kWLD];
  const uint32_t mine = count[cls];
  const int32_t* const list = nodes + (int64_t)cls * n;
  GramTally tally;
  for (uint32_t i = blockIdx.x; i < mine; i += gridDim.x) {
    const int64_t s = list[i];
    gram_node<METRIC, WHOLE, RBM, COM>(S, tile, vs, s, p, merge_mode, snew, sold, cnew[s], cold[s],
                                       meta, pslot, slots, bins, tally);
    __syncthreads();  // the LDS arrays are taken over by the next node
  }
  if (threadIdx.x == 0) {
    uint64_t* cs = counters + (blockIdx.x & (kStripes - 1)) * C_SLOTS;
    if (tally.passed) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_PASSED),
                                (unsigned long long)tally.passed);
    if (tally.overflow) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_OVERFLOW),
                                  (unsigned long long)tally.overflow);
    if (tally.found) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_PROPS),
                               (unsigned long long)tally.found);
    if (tally.evals) atomicAdd(reinterpret_cast<unsigned long long*>(cs + C_EVALS),
                               (unsigned long long)tally.evals);
  }
}

__global__ __launch_bounds__(256) void k_gram_norms(int64_t n, const float* __restrict__ norms,
                                                    NodeMeta* meta) {
  const int64_t s = block_linear() * 256 + threadIdx.x;
  if (s < n) meta[s].norm = (int32_t)__float_as_uint(norms[s]);
}

int compute_units() {
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

}  // namespace

hipError_t launch_gram_norms(const Shape& sh, const DevState& ds, hipStream_t st) {
  static_assert(sizeof(NodeMeta) == 8 && offsetof(NodeMeta, kth) == 0 && offsetof(NodeMeta, norm) == 4,
                "k_join_gram reads a NodeMeta as (kth, norm bits)");
  k_gram_norms<<<grid_blocks((sh.n + 255) / 256), 256, 0, st>>>(sh.n, sh.norms, ds.meta);
  return hipGetLastError();
}

hipError_t launch_join_gram(const Shape& sh, const DevState& ds, bool merge_mode, hipStream_t st) {
  VecSrc vs{sh.vec_a, sh.vec_b, sh.split, sh.d, sh.norms};
  const uint64_t slots = (uint64_t)sh.slots();
  const int mm = merge_mode ? 1 : 0;
  // the nodes with work to do, by class
  hipError_t e = launch_zero_u32(ds.cls_count, kGramClasses, st);
  if (e != hipSuccess) return e;
  k_gram_classify<<<grid_blocks((sh.n + kClassifyNodes - 1) / kClassifyNodes), 256, 0, st>>>(
      sh.n, mm, ds.cnew, ds.cold, ds.cls_nodes, ds.cls_count);
  // one build per class, each with about four sets of resident wavefronts (the lists' lengths
  // are known on the device only) and never more wavefronts than nodes
  const int64_t cap = (int64_t)64 * compute_units();
  const unsigned grid = (unsigned)(sh.n < cap ? sh.n : cap);
#define GNND_GRAM_ARGS vs, sh.n, sh.p, mm, ds.snew, ds.sold, ds.cnew, ds.cold, ds.meta, ds.pslot, \
                       slots, ds.bins, ds.counters, ds.cls_nodes, ds.cls_count
  // (in a merge no node without OLD samples has work to do)
#define GNND_GRAM_CLASSES(M, W)                                                \
  if (!merge_mode) k_join_gram<M, W, 0><<<grid, kWave, 0, st>>>(GNND_GRAM_ARGS); \
  k_join_gram<M, W, 1><<<grid, kWave, 0, st>>>(GNND_GRAM_ARGS);                  \
  k_join_gram<M, W, 2><<<grid, kWave, 0, st>>>(GNND_GRAM_ARGS);                  \
  k_join_gram<M, W, 3><<<grid, kWave, 0, st>>>(GNND_GRAM_ARGS);                  \
  k_join_gram<M, W, 4><<<grid, kWave, 0, st>>>(GNND_GRAM_ARGS);                  \
  k_join_gram<M, W, 5><<<grid, kWave, 0, st>>>(GNND_GRAM_ARGS);                  \
  k_join_gram<M, W, 6><<<grid, kWave, 0, st>>>(GNND_GRAM_ARGS);
#define GNND_GRAM_LAUNCH(M)                      \
  if (sh.d % kWC == 0) {                         \
    GNND_GRAM_CLASSES(M, true)                   \
  } else {                                       \
    GNND_GRAM_CLASSES(M, false)                  \
  }
  switch (sh.metric) {
    case kL2F32: GNND_GRAM_LAUNCH(kL2F32) break;
    case kAngularF32: GNND_GRAM_LAUNCH(kAngularF32) break;
    case kCosineF32: GNND_GRAM_LAUNCH(kCosineF32) break;
    default: return hipErrorInvalidValue;  // no inner-product form for the other metrics
  }
#undef GNND_GRAM_LAUNCH
#undef GNND_GRAM_CLASSES
#undef GNND_GRAM_ARGS
  return hipGetLastError();
}

}  // namespace gnnd
