// Reverse-neighbour candidates (Sec. 4.1) grouped by target without global
// atomics.  Device-wide atomics run at a fixed ~27 G/s (12 G/s when the old
// value is needed), which made them the cost of the sampling stage, so the
// transpose "s samples v  ->  s is a candidate of v" is done as a two-level
// counting sort instead:
//   1. k_fwd_count   - forward sampling of every list (first p NEW / first p
//                      OLD entries, sampled NEW flagged OLD); per workgroup an
//                      LDS histogram of the targets' buckets (bucket = target id
//                      >> tb), kept as one column of a (bucket x workgroup)
//                      matrix.
//   2. k_wg_scan     - exclusive scan along the matrix rows: every workgroup's
//                      run start inside every bucket, and the bucket sizes.
//      k_bucket_scan - exclusive scan of the <= 4096 bucket sizes per kind.
//   3. k_fwd_scatter_staged - every workgroup writes its (target, source)
//                      edges into its runs, sorted by bucket in LDS first.
//   4. k_bucket_csr  - one workgroup per bucket: LDS counters per target,
//                      block scan = the targets' segment offsets, second sweep
//                      places the sources.  Buckets are in target order, so the
//                      result is the same CSR a global scan would give.
// The loops over rows and edges keep several independent loads in flight per
// thread; with one load per trip they are bound by memory latency.
#include "device_utils.hpp"
#include "kernels.hpp"

namespace gnnd {

constexpr int kSB = 256;
constexpr int kMaxBuckets = 4096;
constexpr int kCsrBlock = 1024;

struct BucketGeom {
  int tb;         // log2(targets per bucket)
  int nb;         // buckets
  int rows_per_wg;
};

// Forward sampling of one list by one wavefront; returns this lane's sampled id
// (or -1) for each kind and writes the forward parts of the sample rows.
__device__ inline void forward_sample_row(int64_t s, int64_t n, int k, int p, uint64_t* G,
                                          int32_t* snew, int32_t* sold, int32_t* cnew,
                                          int32_t* cold, int lane, uint64_t e, int32_t& v_new,
                                          int32_t& v_old) {
  // e = this lane's entry of the row (lanes >= k: anything)
  // entries numbered beyond n are frozen leftovers of an earlier merge: not sampled
  const bool valid = lane < k && (int64_t)entry_id(e) < n;
  const bool isnew = valid && (e & 1ull);
  const bool isold = valid && !(e & 1ull);
  const uint64_t mn = __ballot(isnew), mo = __ballot(isold);
  const int rn = __popcll(mn & lanes_below(lane)), ro = __popcll(mo & lanes_below(lane));
  const int32_t id = (int32_t)entry_id(e);
  const int L = 2 * p;
  v_new = v_old = -1;
  if (isnew && rn < p) {
    snew[s * L + rn] = id;
    G[s * k + lane] = e & ~1ull;
    v_new = id;
  }
  if (isold && ro < p) {
    sold[s * L + ro] = id;
    v_old = id;
  }
  const int cn = __popcll(mn) < p ? __popcll(mn) : p, co = __popcll(mo) < p ? __popcll(mo) : p;
  // the rest of the forward part reads "nothing", so that the scatter pass needs no counts
  if (lane >= cn && lane < p) snew[s * L + lane] = -1;
  if (lane >= co && lane < p) sold[s * L + lane] = -1;
  if (lane == 0) {
    cnew[s] = cn;
    cold[s] = co;
  }
}

// The same for a list of 65..128 entries, two per lane (e0 = entry lane, e1 =
// entry lane + 64 or 0): ranks run through the first register, then the second.
__device__ inline void forward_sample_row_wide(int64_t s, int64_t n, int k, int p, uint64_t* G,
                                               int32_t* snew, int32_t* sold, int32_t* cnew,
                                               int32_t* cold, int lane, uint64_t e0, uint64_t e1,
                                               int32_t (&v_new)[2], int32_t (&v_old)[2]) {
  const uint64_t e[2] = {e0, e1};
  uint64_t mn[2], mo[2];
  bool isnew[2], isold[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const bool valid = lane + r * kWave < k && (int64_t)entry_id(e[r]) < n;
    isnew[r] = valid && (e[r] & 1ull);
    isold[r] = valid && !(e[r] & 1ull);
    mn[r] = __ballot(isnew[r]);
    mo[r] = __ballot(isold[r]);
  }
  const int L = 2 * p;
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int rn = (r ? __popcll(mn[0]) : 0) + __popcll(mn[r] & lanes_below(lane));
    const int ro = (r ? __popcll(mo[0]) : 0) + __popcll(mo[r] & lanes_below(lane));
    const int32_t id = (int32_t)entry_id(e[r]);
    v_new[r] = v_old[r] = -1;
    if (isnew[r] && rn < p) {
      snew[s * L + rn] = id;
      G[s * k + r * kWave + lane] = e[r] & ~1ull;
      v_new[r] = id;
    }
    if (isold[r] && ro < p) {
      sold[s * L + ro] = id;
      v_old[r] = id;
    }
  }
  const int tn = __popcll(mn[0]) + __popcll(mn[1]), to = __popcll(mo[0]) + __popcll(mo[1]);
  const int cn = tn < p ? tn : p, co = to < p ? to : p;
  if (lane >= cn && lane < p) snew[s * L + lane] = -1;
  if (lane >= co && lane < p) sold[s * L + lane] = -1;
  if (lane == 0) {
    cnew[s] = cn;
    cold[s] = co;
  }
}

template <bool WIDE>
__global__ __launch_bounds__(kSB) void k_fwd_count(int64_t n, int k, int p, BucketGeom g,
                                                   uint64_t* G, int32_t* snew, int32_t* sold,
                                                   int32_t* cnew, int32_t* cold,
                                                   uint32_t* wg_hist) {
  __shared__ uint32_t hist[2 * kMaxBuckets];
  for (int i = threadIdx.x; i < 2 * g.nb; i += kSB) hist[i] = 0;
  __syncthreads();
  const int lane = lane_id(), wave = wave_id();
  const int64_t row0 = (int64_t)blockIdx.x * g.rows_per_wg;
  const int64_t row1 = row0 + g.rows_per_wg < n ? row0 + g.rows_per_wg : n;
  constexpr int kRowsAtOnce = 4;  // rows in flight per wavefront
  constexpr int kStep = kRowsAtOnce * (kSB / kWave);
  for (int64_t s0 = row0 + wave; s0 < row1; s0 += kStep) {
    uint64_t e[kRowsAtOnce], e1[kRowsAtOnce];
#pragma unroll
    for (int r = 0; r < kRowsAtOnce; ++r) {
      const int64_t s = s0 + r * (kSB / kWave);
      e[r] = (s < row1 && lane < k) ? G[s * k + lane] : 0ull;
      if (WIDE) e1[r] = (s < row1 && lane + kWave < k) ? G[s * k + kWave + lane] : 0ull;
    }
#pragma unroll
    for (int r = 0; r < kRowsAtOnce; ++r) {
      const int64_t s = s0 + r * (kSB / kWave);
      if (s >= row1) break;
      if (WIDE) {
        int32_t vn[2], vo[2];
        forward_sample_row_wide(s, n, k, p, G, snew, sold, cnew, cold, lane, e[r], e1[r], vn, vo);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          if (vn[q] >= 0) atomicAdd(&hist[vn[q] >> g.tb], 1u);
          if (vo[q] >= 0) atomicAdd(&hist[g.nb + (vo[q] >> g.tb)], 1u);
        }
      } else {
        int32_t vn, vo;
        forward_sample_row(s, n, k, p, G, snew, sold, cnew, cold, lane, e[r], vn, vo);
        if (vn >= 0) atomicAdd(&hist[vn >> g.tb], 1u);
        if (vo >= 0) atomicAdd(&hist[g.nb + (vo >> g.tb)], 1u);
      }
    }
  }
  __syncthreads();
  // column blockIdx.x of the (bucket x workgroup) count matrix
  for (int i = threadIdx.x; i < 2 * g.nb; i += kSB) wg_hist[(size_t)i * gridDim.x + blockIdx.x] = hist[i];
}

// Exclusive scan along every row of the (bucket x workgroup) count matrix: the
// entry of workgroup w becomes the start of w's run inside the bucket, the row
// total the bucket's size.  One wavefront per row - no atomics, and the edge
// order inside a bucket no longer depends on timing.
__global__ __launch_bounds__(kSB) void k_wg_scan(int W, int rows, uint32_t* wg_hist,
                                                 uint32_t* bcnt) {
  const int c = blockIdx.x * (kSB / kWave) + wave_id();
  if (c >= rows) return;
  const int lane = lane_id();
  uint32_t* row = wg_hist + (size_t)c * W;
  constexpr int kChunks = 4;  // chunks of 64 entries in flight
  uint32_t carry = 0;
  for (int w0 = 0; w0 < W; w0 += kChunks * kWave) {
    uint32_t v[kChunks];
#pragma unroll
    for (int r = 0; r < kChunks; ++r) {
      const int w = w0 + r * kWave + lane;
      v[r] = w < W ? row[w] : 0u;
    }
#pragma unroll
    for (int r = 0; r < kChunks; ++r) {
      const int w = w0 + r * kWave + lane;
      uint32_t inc = v[r];
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t o = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += o;
      }
      if (w < W) row[w] = carry + inc - v[r];
      carry += __shfl(inc, kWave - 1, kWave);
    }
  }
  if (lane == 0) bcnt[c] = carry;
}

// boff[kind][0..nb] = exclusive scan of the bucket sizes bcnt[kind][0..nb).
__global__ __launch_bounds__(kCsrBlock) void k_bucket_scan(int nb, const uint32_t* bcnt,
                                                           uint64_t* boff) {
  __shared__ uint64_t part[kCsrBlock];
  for (int kind = 0; kind < 2; ++kind) {
    const uint32_t* c = bcnt + kind * nb;
    uint64_t* o = boff + kind * (nb + 1);
    const int per = (nb + kCsrBlock - 1) / kCsrBlock;
    const int lo = threadIdx.x * per;
    uint64_t sum = 0;
    for (int i = lo; i < lo + per && i < nb; ++i) sum += c[i];
    part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
      uint64_t run = 0;
      for (int i = 0; i < kCsrBlock; ++i) {
        uint64_t v = part[i];
        part[i] = run;
        run += v;
      }
      o[nb] = run;
    }
    __syncthreads();
    uint64_t run = part[threadIdx.x];
    for (int i = lo; i < lo + per && i < nb; ++i) {
      o[i] = run;
      run += c[i];
    }
    __syncthreads();
  }
}

// Scatter pass.  A workgroup of 1024 threads takes its rows in batches of 256,
// sorts a batch's edges of one kind by bucket in LDS (count, scan, place), and
// copies them out in that order, so that the part of a batch that goes to one
// bucket leaves as one contiguous piece instead of one 8-byte store per edge to
// as many places (0.50 -> 0.24 ms per million nodes).
// PW threads serve a row (its up to PW forward samples of one kind): 32 for p <= 32, 64 beyond.
constexpr int kStBlock = 1024;
constexpr int kStEdges = 256 * 32;           // edges per batch: 256 rows of 32, or 128 rows of 64
constexpr int kStPasses = 8;                 // passes of kStBlock / PW rows make a batch

// PACKED: an edge leaves as one 32-bit word, (target inside its bucket) << (32 - tb) | source,
// which the sources of up to 2^(32 - tb) nodes fit; otherwise as (target, source).
template <int PW, bool PACKED>
__global__ __launch_bounds__(kStBlock) void k_fwd_scatter_staged(
    int64_t n, int p, BucketGeom g, const int32_t* snew, const int32_t* sold,
    const uint32_t* wg_hist, const uint64_t* boff, uint2* edges_new, uint2* edges_old) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  uint32_t* cursor = lds;               // 2 nb: where this workgroup writes next, per kind and bucket
  uint32_t* cnt = cursor + 2 * g.nb;    // nb: edges of the batch per bucket
  uint32_t* off = cnt + g.nb;           // nb + 1: their exclusive scan
  uint32_t* wsum = off + g.nb + 1;      // 16 wave totals of the scan
  uint2* stage = reinterpret_cast<uint2*>(lds + ((4 * g.nb + 17 + 3) & ~3));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 2 * g.nb; i += kStBlock) {
    const uint64_t bucket_start = i < g.nb ? boff[i] : boff[i + 1];
    cursor[i] = (uint32_t)bucket_start + wg_hist[(size_t)i * gridDim.x + blockIdx.x];
  }
  const int L = 2 * p;
  const int64_t row0 = (int64_t)blockIdx.x * g.rows_per_wg;
  const int64_t row1 = row0 + g.rows_per_wg < n ? row0 + g.rows_per_wg : n;
  const int per = (g.nb + kStBlock - 1) / kStBlock;  // buckets per thread in the scan (<= 4)
  constexpr int kRowsPerPass = kStBlock / PW, kStRows = kStPasses * kRowsPerPass;
  static_assert(kStRows * PW == kStEdges, "a batch fills the staging area");
  const int sub = tid & (PW - 1), rsel = tid / PW;     // entry of a row, row of a pass
  for (int64_t b0 = row0; b0 < row1; b0 += kStRows) {
    for (int kind = 0; kind < 2; ++kind) {
      const int32_t* list = kind ? sold : snew;
      uint2* edges = kind ? edges_old : edges_new;
      for (int i = tid; i < g.nb; i += kStBlock) cnt[i] = 0;
      __syncthreads();
      int32_t v[kStPasses];
      uint32_t rank[kStPasses];
#pragma unroll
      for (int q = 0; q < kStPasses; ++q) {
        const int64_t s = b0 + q * kRowsPerPass + rsel;
        v[q] = (s < row1 && sub < p) ? list[s * L + sub] : -1;
      }
#pragma unroll
      for (int q = 0; q < kStPasses; ++q)
        rank[q] = v[q] >= 0 ? atomicAdd(&cnt[(uint32_t)v[q] >> g.tb], 1u) : 0u;
      __syncthreads();
      // exclusive scan of cnt into off: `per` consecutive buckets per thread
      uint32_t mine = 0;
      for (int i = 0; i < per; ++i) {
        const int b = tid * per + i;
        mine += b < g.nb ? cnt[b] : 0u;
      }
      uint32_t inc = mine;
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t t = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += t;
      }
      if (lane == kWave - 1) wsum[wave] = inc;
      __syncthreads();
      uint32_t before = 0;
      for (int w = 0; w < wave; ++w) before += wsum[w];
      uint32_t run = before + inc - mine;
      for (int i = 0; i < per; ++i) {
        const int b = tid * per + i;
        if (b < g.nb) {
          off[b] = run;
          run += cnt[b];
        }
      }
      if (tid == kStBlock - 1) off[g.nb] = run;
      __syncthreads();
#pragma unroll
      for (int q = 0; q < kStPasses; ++q)
        if (v[q] >= 0) {
          const int64_t s = b0 + q * kRowsPerPass + rsel;
          stage[off[(uint32_t)v[q] >> g.tb] + rank[q]] = make_uint2((uint32_t)v[q], (uint32_t)s);
        }
      __syncthreads();
      const uint32_t total = off[g.nb];
      for (uint32_t i = tid; i < total; i += kStBlock) {
        const uint2 rec = stage[i];
        const uint32_t b = rec.x >> g.tb;
        const uint32_t at = cursor[kind * g.nb + b] + (i - off[b]);
        if (PACKED)
          reinterpret_cast<uint32_t*>(edges)[at] =
              ((rec.x & ((1u << g.tb) - 1u)) << (32 - g.tb)) | rec.y;
        else
          edges[at] = rec;
      }
      __syncthreads();
      for (int i = tid; i < g.nb; i += kStBlock) cursor[kind * g.nb + i] += cnt[i];
      // (the next round's first barrier orders these updates before their use)
    }
  }
}

static size_t staged_lds_bytes(const BucketGeom& g) {
  return (size_t)((4 * g.nb + 17 + 3) & ~3) * 4 + (size_t)kStEdges * 8;
}

// One workgroup per (bucket, kind): counting sort of the bucket's edges by
// target.  LDS holds one counter per target of the bucket (dynamic size).
template <bool PACKED>
__global__ __launch_bounds__(kCsrBlock) void k_bucket_csr(int64_t n, BucketGeom g,
                                                          const uint64_t* boff,
                                                          const uint2* edges_new,
                                                          const uint2* edges_old,
                                                          uint64_t* roff_new, uint64_t* roff_old,
                                                          int32_t* csr_new, int32_t* csr_old) {
  extern __shared__ uint32_t cnt[];  // 2^tb counters, then running offsets
  __shared__ uint32_t part[kCsrBlock];
  const int kind = blockIdx.y;
  const int b = blockIdx.x;
  const uint64_t* bo = boff + kind * (g.nb + 1);
  const uint2* edges = kind ? edges_old : edges_new;
  uint64_t* roff = kind ? roff_old : roff_new;
  int32_t* csr = kind ? csr_old : csr_new;
  const uint64_t beg = bo[b], end = bo[b + 1];
  const int T = 1 << g.tb;
  const uint32_t mask = (uint32_t)T - 1u;
  for (int i = threadIdx.x; i < T; i += kCsrBlock) cnt[i] = 0;
  __syncthreads();
  constexpr int kAtOnce = 8;  // edges in flight per thread
  const uint32_t* const words = reinterpret_cast<const uint32_t*>(edges);
  const int sh = 32 - g.tb;  // packed edge: target inside the bucket above, source below
  for (uint64_t e0 = beg + threadIdx.x; e0 < end; e0 += kAtOnce * kCsrBlock) {
    uint32_t t[kAtOnce];
#pragma unroll
    for (int r = 0; r < kAtOnce; ++r) {
      const uint64_t e = e0 + (uint64_t)r * kCsrBlock;
      t[r] = e < end ? (PACKED ? words[e] >> sh : edges[e].x & mask) : 0xffffffffu;
    }
#pragma unroll
    for (int r = 0; r < kAtOnce; ++r)
      if (t[r] != 0xffffffffu) atomicAdd(&cnt[t[r]], 1u);
  }
  __syncthreads();
  // exclusive scan over the T counters: T / 1024 consecutive counters per thread
  const int per = T / kCsrBlock;  // T >= 4096
  const int lo = threadIdx.x * per;
  uint32_t sum = 0;
  for (int i = 0; i < per; ++i) sum += cnt[lo + i];
  part[threadIdx.x] = sum;
  __syncthreads();
  if (threadIdx.x < kWave) {  // scan of the 1024 partial sums by one wavefront, 16 each
    uint32_t local[kCsrBlock / kWave];
    uint32_t s2 = 0;
    for (int i = 0; i < kCsrBlock / kWave; ++i) {
      local[i] = s2;
      s2 += part[threadIdx.x * (kCsrBlock / kWave) + i];
    }
    uint32_t inc = s2;
    for (int off = 1; off < kWave; off <<= 1) {
      uint32_t o = __shfl_up(inc, off, kWave);
      if ((int)threadIdx.x >= off) inc += o;
    }
    const uint32_t before = inc - s2;
    for (int i = 0; i < kCsrBlock / kWave; ++i)
      part[threadIdx.x * (kCsrBlock / kWave) + i] = before + local[i];
  }
  __syncthreads();
  uint32_t run = part[threadIdx.x];
  const int64_t first = (int64_t)b << g.tb;
  for (int i = 0; i < per; ++i) {
    const uint32_t c = cnt[lo + i];
    cnt[lo + i] = run;  // start of the target's segment inside the bucket
    if (first + lo + i < n) roff[first + lo + i] = beg + run;
    run += c;
  }
  if (b == g.nb - 1 && threadIdx.x == 0) roff[n] = bo[g.nb];
  __syncthreads();
  for (uint64_t e0 = beg + threadIdx.x; e0 < end; e0 += kAtOnce * kCsrBlock) {
    uint2 ed[kAtOnce];  // (target inside the bucket, source); target 0xffffffff: none
#pragma unroll
    for (int r = 0; r < kAtOnce; ++r) {
      const uint64_t e = e0 + (uint64_t)r * kCsrBlock;
      ed[r] = make_uint2(0xffffffffu, 0u);
      if (e < end) {
        if (PACKED) {
          const uint32_t w = words[e];
          ed[r] = make_uint2(w >> sh, w & ((1u << sh) - 1u));
        } else {
          const uint2 x = edges[e];
          ed[r] = make_uint2(x.x & mask, x.y);
        }
      }
    }
#pragma unroll
    for (int r = 0; r < kAtOnce; ++r)
      if (ed[r].x != 0xffffffffu) {
        const uint32_t pos = atomicAdd(&cnt[ed[r].x], 1u);
        csr[beg + pos] = (int32_t)ed[r].y;
      }
  }
}

// The bucket layout for n <= 2^27 targets: at most 4096 buckets of 2^tb <= 2^15
// targets (one workgroup's LDS counts a bucket's targets).
static BucketGeom bucket_geom(int64_t n) {
  BucketGeom g{10, 0, 256};
  while (((n + (1ll << g.tb) - 1) >> g.tb) > kMaxBuckets) ++g.tb;
  g.nb = (int)((n + (1ll << g.tb) - 1) >> g.tb);
  g.rows_per_wg = g.nb > 256 ? g.nb : 256;
  return g;
}

hipError_t launch_sample_buckets(const Shape& sh, const DevState& ds, hipStream_t st) {
  const BucketGeom g = bucket_geom(sh.n);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_bucket_csr<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 4 << 15);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_bucket_csr<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 4 << 15);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  uint32_t* bcnt = ds.bk_cnt;
  uint64_t* boff = ds.bk_off;
  uint2* edges_new = reinterpret_cast<uint2*>(ds.bins);
  uint2* edges_old = edges_new + sh.n * sh.p;
  // per-workgroup bucket histograms, behind the edges in the same (still unused) array
  uint32_t* wg_hist = reinterpret_cast<uint32_t*>(edges_old + sh.n * sh.p);
  const unsigned grid = (unsigned)((sh.n + g.rows_per_wg - 1) / g.rows_per_wg);
  if (sh.k > kWave)
    k_fwd_count<true><<<grid, kSB, 0, st>>>(sh.n, sh.k, sh.p, g, ds.G, ds.snew, ds.sold, ds.cnew,
                                            ds.cold, wg_hist);
  else
    k_fwd_count<false><<<grid, kSB, 0, st>>>(sh.n, sh.k, sh.p, g, ds.G, ds.snew, ds.sold, ds.cnew,
                                             ds.cold, wg_hist);
  k_wg_scan<<<(unsigned)((2 * g.nb + kSB / kWave - 1) / (kSB / kWave)), kSB, 0, st>>>(
      (int)grid, 2 * g.nb, wg_hist, bcnt);
  k_bucket_scan<<<1, kCsrBlock, 0, st>>>(g.nb, bcnt, boff);
  static bool staged_attr = false;
  if (!staged_attr) {
    hipError_t e = hipSuccess;
    const void* kernels[4] = {reinterpret_cast<const void*>(k_fwd_scatter_staged<32, false>),
                              reinterpret_cast<const void*>(k_fwd_scatter_staged<32, true>),
                              reinterpret_cast<const void*>(k_fwd_scatter_staged<64, false>),
                              reinterpret_cast<const void*>(k_fwd_scatter_staged<64, true>)};
    for (int i = 0; i < 4 && e == hipSuccess; ++i)
      e = hipFuncSetAttribute(kernels[i], hipFuncAttributeMaxDynamicSharedMemorySize, 144 << 10);
    if (e != hipSuccess) return e;
    staged_attr = true;
  }
  // one 32-bit word per edge where the source ids fit beside the target's place in its bucket
  const bool packed = sh.n <= ((int64_t)1 << (32 - g.tb));
#define GNND_SCATTER(PW, PK)                                                            \
  k_fwd_scatter_staged<PW, PK><<<grid, kStBlock, staged_lds_bytes(g), st>>>(            \
      sh.n, sh.p, g, ds.snew, ds.sold, wg_hist, boff, edges_new, edges_old)
  if (sh.p <= 32) {
    if (packed) GNND_SCATTER(32, true);
    else GNND_SCATTER(32, false);
  } else {
    if (packed) GNND_SCATTER(64, true);
    else GNND_SCATTER(64, false);
  }
#undef GNND_SCATTER
  if (packed)
    k_bucket_csr<true><<<dim3((unsigned)g.nb, 2), kCsrBlock, (size_t)4 << g.tb, st>>>(
        sh.n, g, boff, edges_new, edges_old, ds.roff_new, ds.roff_old, ds.csr_new, ds.csr_old);
  else
    k_bucket_csr<false><<<dim3((unsigned)g.nb, 2), kCsrBlock, (size_t)4 << g.tb, st>>>(
        sh.n, g, boff, edges_new, edges_old, ds.roff_new, ds.roff_old, ds.csr_new, ds.csr_old);
  return hipGetLastError();
}

}  // namespace gnnd
