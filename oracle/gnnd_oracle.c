/*
 * CPU oracle for GPU NN-Descent (GNND) and the GPU graph merge (GGM).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, sequential statement
 * of what one GNND iteration and one GGM merge compute.  Nothing in the product
 * library links against it or calls it; only the test-suite, the smoke check and
 * the CPU-baseline leg of the benchmark do.  It shares no code, header, table or
 * constant generator with the HIP implementation.
 *
 * Each function cites the passage of the paper it follows (arxiv 2103.15386:
 * "Alg. 1" = ConstructKNNGraph, "Alg. 2" = GetNearestObject, "Alg. 3" = GGM,
 * "Sec. 4.1/4.2/4.3/5.1", "Eq. 1-2" = thread-to-pair map, "Eq. 4" = Recall@k).
 * Where the paper leaves a choice open the reading taken is stated in the
 * comment of the function.
 *
 * Pins (tests/test_oracle_*.py): every function below is checked against
 * something other than itself - published splitmix64 outputs, numpy float64
 * brute force, closed special cases (k = n-1; 1-d points on a line; candidate
 * count below the cap; n2 = floor(k/2) for the merge), set-function identities
 * and monotonicity invariants.  What stays unpinned: the recall values the
 * iteration reaches on the large synthetic workloads ("parity unpinned": only
 * this oracle defines them).
 *
 * Distances are held as double in the graph arrays: a float32 or int32 distance
 * converts to double exactly, so one comparison routine serves all metrics while
 * the decisions are still those of the metric's own precision.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { OG_L2SQ_F32 = 0, OG_ANGULAR_F32 = 1, OG_L2SQ_U8 = 2, OG_CHI2_F32 = 3, OG_COSINE_F32 = 4 };
enum { OG_TAG_INIT = 1, OG_TAG_REV_NEW = 2, OG_TAG_REV_OLD = 3, OG_TAG_MERGE = 4 };
enum { OG_HASH_ATTEMPTS = 256 };

/* ------------------------------------------------------------------------- */
/* Counter-based random numbers.  The paper only says "random objects"
 * (Alg. 1, first loop) and treats the racing reverse appends as "random
 * sampling" (Sec. 4.1); it fixes no generator.  Reading: a stateless hash of
 * (seed, purpose tag, three counters) built from the splitmix64 output mixer
 * (Steele/Lea/Flood; Vigna's public-domain splitmix64), so any evaluation
 * order gives the same draws. */
uint64_t og_mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xbf58476d1ce4e5b9ULL;
  z ^= z >> 27;
  z *= 0x94d049bb133111ebULL;
  z ^= z >> 31;
  return z;
}

uint64_t og_hash(uint64_t seed, uint32_t tag, uint32_t a, uint32_t b, uint32_t c) {
  uint64_t h = og_mix64(seed + 0x9e3779b97f4a7c15ULL * ((uint64_t)tag + 1));
  h = og_mix64(h ^ (((uint64_t)a << 32) | (uint64_t)b));
  h = og_mix64(h + (uint64_t)c);
  return h;
}

/* Map the upper 32 bits of a hash onto [0, n) by multiply-high. */
uint32_t og_bounded(uint64_t h, uint32_t n) {
  return (uint32_t)(((h >> 32) * (uint64_t)n) >> 32);
}

/* ------------------------------------------------------------------------- */
/* Distance between stored vectors i and j.  The paper computes "the l2-norm"
 * between sub-vectors phase by phase and aggregates (Sec. 4.2); single
 * precision is implied (one float per shared-memory cell).  Reading: squared
 * L2 accumulated in float32 with one fused multiply-add per dimension, in
 * dimension order; angular = 1 - dot (float32, same order); bytes give an
 * exact int32 squared L2.  Two builds of the float loops (hardware FMA or
 * libm's exact fmaf) return identical bits. */
__attribute__((target_clones("fma", "default"))) static float l2sq_f32(const float* a,
                                                                      const float* b, int d) {
  float acc = 0.0f;
  for (int j = 0; j < d; ++j) {
    float diff = a[j] - b[j];
    acc = fmaf(diff, diff, acc);
  }
  return acc;
}

__attribute__((target_clones("fma", "default"))) static float dot_f32(const float* a,
                                                                     const float* b, int d) {
  float acc = 0.0f;
  for (int j = 0; j < d; ++j) acc = fmaf(a[j], b[j], acc);
  return acc;
}

/* Chi-square distance of two non-negative vectors (Sec. 4.2 names it next to the
 * l2-norm as a metric the tile kernel can evaluate): sum over the dimensions of
 * (a - b)^2 / (a + b), a dimension with a + b = 0 adding nothing.  Reading: float32,
 * dimension order, every operation rounded on its own (no fused multiply-add;
 * the build switches contraction off). */
static float chi2_f32(const float* a, const float* b, int d) {
  float acc = 0.0f;
  for (int j = 0; j < d; ++j) {
    const float diff = a[j] - b[j];
    const float sum = a[j] + b[j];
    if (sum > 0.0f) {
      const float sq = diff * diff;
      acc = acc + sq / sum;
    }
  }
  return acc;
}

/* Cosine distance of vectors that are not unit length (Sec. 1: the method keeps
 * NN-Descent's genericness over distance metrics; this one needs the two norms
 * besides the inner product):
 * 1 - a.b / sqrt(|a|^2 |b|^2).  Reading: float32; the inner product and the two
 * squared norms each accumulated with one fused multiply-add per dimension, in
 * dimension order (a squared norm is a property of its vector alone); product,
 * square root, quotient and difference each rounded on their own; a zero vector
 * is at distance 1 from everything. */
static float cosine_f32(const float* a, const float* b, int d) {
  const float dot = dot_f32(a, b, d);
  const float na = dot_f32(a, a, d);
  const float nb = dot_f32(b, b, d);
  const float den = sqrtf(na * nb);
  return den > 0.0f ? 1.0f - dot / den : 1.0f;
}

double og_distance(int metric, int d, const void* vec, int64_t i, int64_t j) {
  if (metric == OG_COSINE_F32) {
    const float* x = (const float*)vec;
    return (double)cosine_f32(x + i * d, x + j * d, d);
  }
  if (metric == OG_CHI2_F32) {
    const float* x = (const float*)vec;
    return (double)chi2_f32(x + i * d, x + j * d, d);
  }
  if (metric == OG_L2SQ_F32) {
    const float* x = (const float*)vec;
    return (double)l2sq_f32(x + i * d, x + j * d, d);
  } else if (metric == OG_ANGULAR_F32) {
    const float* x = (const float*)vec;
    float dot = dot_f32(x + i * d, x + j * d, d);
    return (double)(1.0f - dot);
  } else {
    const uint8_t* x = (const uint8_t*)vec;
    const uint8_t* a = x + i * d;
    const uint8_t* b = x + j * d;
    int32_t acc = 0;
    for (int q = 0; q < d; ++q) {
      int32_t diff = (int32_t)a[q] - (int32_t)b[q];
      acc += diff * diff;
    }
    return (double)acc;
  }
}

/* (distance, id) lexicographic order: the tie-break used everywhere. */
static int closer(double d1, int32_t id1, double d2, int32_t id2) {
  return d1 < d2 || (d1 == d2 && id1 < id2);
}

typedef struct {
  double d;
  int32_t id;
  uint8_t isnew;
  uint8_t fresh; /* 1 = came from a proposal in this update */
} entry_t;

static int entry_cmp(const void* pa, const void* pb) {
  const entry_t* a = (const entry_t*)pa;
  const entry_t* b = (const entry_t*)pb;
  if (closer(a->d, a->id, b->d, b->id)) return -1;
  if (closer(b->d, b->id, a->d, a->id)) return 1;
  /* same (distance, id): an entry already in the list goes first */
  return (int)a->fresh - (int)b->fresh;
}

/* ------------------------------------------------------------------------- */
/* Exact k-NN by exhaustive search ("each sample is compared against the rest
 * of the dataset", Sec. 6): for every query node the K closest other nodes by
 * (distance, id). */
void og_bruteforce(const void* vec, int64_t n, int d, int metric, const int32_t* queries,
                   int64_t nq, int K, int32_t* out_ids, double* out_dist) {
#pragma omp parallel for schedule(dynamic, 4)
  for (int64_t q = 0; q < nq; ++q) {
    int32_t s = queries[q];
    int32_t* bi = out_ids + q * K;
    double* bd = out_dist + q * K;
    int have = 0;
    for (int64_t c = 0; c < n; ++c) {
      if (c == s) continue;
      double dist = og_distance(metric, d, vec, s, c);
      if (have == K && !closer(dist, (int32_t)c, bd[K - 1], bi[K - 1])) continue;
      int pos = have < K ? have : K - 1;
      while (pos > 0 && closer(dist, (int32_t)c, bd[pos - 1], bi[pos - 1])) {
        bd[pos] = bd[pos - 1];
        bi[pos] = bi[pos - 1];
        --pos;
      }
      bd[pos] = dist;
      bi[pos] = (int32_t)c;
      if (have < K) ++have;
    }
    for (int r = have; r < K; ++r) {
      bi[r] = -1;
      bd[r] = INFINITY;
    }
  }
}

/* ------------------------------------------------------------------------- */
/* Draw `count` distinct ids for node s out of [0, n_range) + base.  Slot j takes
 * og_hash(seed, tag, s, j, attempt) mapped onto the range, attempt = 0, 1, ...
 * until the id is neither `forbid` nor one drawn for an earlier slot; after
 * OG_HASH_ATTEMPTS failed attempts it steps to the next id (cyclically) until
 * one is free, which always ends because count <= number of allowed ids. */
static void draw_distinct_from(uint64_t seed, uint32_t tag, uint32_t s, int slot0, int count,
                               uint32_t n_range, int32_t base, int32_t forbid, int32_t* out);
static void draw_distinct(uint64_t seed, uint32_t tag, uint32_t s, int count, uint32_t n_range,
                          int32_t base, int32_t forbid, int32_t* out) {
  draw_distinct_from(seed, tag, s, 0, count, n_range, base, forbid, out);
}
/* The same with the slots numbered slot0, slot0 + 1, ... in the hash (several groups of
 * slots of one node, each distinct within itself). */
static void draw_distinct_from(uint64_t seed, uint32_t tag, uint32_t s, int slot0, int count,
                               uint32_t n_range, int32_t base, int32_t forbid, int32_t* out) {
  for (int j = 0; j < count; ++j) {
    uint32_t cand = 0;
    int ok = 0;
    for (uint32_t attempt = 0; attempt < OG_HASH_ATTEMPTS && !ok; ++attempt) {
      cand = og_bounded(og_hash(seed, tag, s, (uint32_t)(slot0 + j), attempt), n_range);
      ok = ((int32_t)cand + base != forbid);
      for (int e = 0; e < j && ok; ++e) ok = (out[e] != (int32_t)cand + base);
    }
    while (!ok) {
      cand = (cand + 1 == n_range) ? 0 : cand + 1;
      ok = ((int32_t)cand + base != forbid);
      for (int e = 0; e < j && ok; ++e) ok = (out[e] != (int32_t)cand + base);
    }
    out[j] = (int32_t)cand + base;
  }
}

/* Alg. 1, first parallel loop: random neighbours, sorted ascending, all NEW.
 * Reading: the listing says "p random objects" but the list has fixed degree k
 * (Sec. 4, first paragraphs; Sec. 3.1 step 1 says k random neighbours), so k
 * distinct ids other than s are drawn; "ascending" = by (distance, id). */
static void init_row(const void* vec, int64_t n, int d, int k, int metric, uint64_t seed,
                     int64_t s, entry_t* row, int32_t* draw, int32_t* ids, double* dist,
                     uint8_t* isnew) {
  draw_distinct(seed, OG_TAG_INIT, (uint32_t)s, k, (uint32_t)n, 0, (int32_t)s, draw);
  for (int j = 0; j < k; ++j) {
    row[j].id = draw[j];
    row[j].d = og_distance(metric, d, vec, s, draw[j]);
    row[j].isnew = 1;
    row[j].fresh = 0;
  }
  qsort(row, (size_t)k, sizeof(entry_t), entry_cmp);
  for (int j = 0; j < k; ++j) {
    ids[j] = row[j].id;
    dist[j] = row[j].d;
    isnew[j] = 1;
  }
}

/* Rows are independent of each other, so the loop may run on several threads. */
void og_init_random(const void* vec, int64_t n, int d, int k, int metric, uint64_t seed,
                    int32_t* ids, double* dist, uint8_t* isnew) {
#pragma omp parallel
  {
    entry_t* row = (entry_t*)malloc(sizeof(entry_t) * (size_t)k);
    int32_t* draw = (int32_t*)malloc(sizeof(int32_t) * (size_t)k);
#pragma omp for schedule(static)
    for (int64_t s = 0; s < n; ++s)
      init_row(vec, n, d, k, metric, seed, s, row, draw, ids + s * k, dist + s * k,
               isnew + s * k);
    free(row);
    free(draw);
  }
}

/* Segmented lists (Sec. 4.3, "Multiple Spinlocks"): a list of k = 32 m entries is kept as
 * m = k / 32 segments of 32 entries, object v can only live in segment v % m, and when an
 * iteration is over the segments are merged into one ascending list.  Reading for the
 * first loop of Alg. 1 (the paper does not say how a segmented list starts): every segment
 * starts with 32 distinct random objects of its own residue class (other than s), drawn
 * like the plain list - slot 32 r + j of node s takes the class member number
 * hash(seed, INIT, s, 32 r + j, attempt) mapped onto the class size; the list is handed out
 * merged, ascending by (distance, id), all NEW.  Every class must have more than 32
 * members (n >= 33 m + m suffices).  With m = 1 this is og_init_random with k = 32. */
void og_init_random_segmented(const void* vec, int64_t n, int d, int k, int metric, uint64_t seed,
                              int32_t* ids, double* dist, uint8_t* isnew) {
  const int m = k / 32;
  entry_t* row = (entry_t*)malloc(sizeof(entry_t) * (size_t)k);
  int32_t* draw = (int32_t*)malloc(sizeof(int32_t) * 32);
  for (int64_t s = 0; s < n; ++s) {
    for (int r = 0; r < m; ++r) {
      const uint32_t members = (uint32_t)((n - r + m - 1) / m);  /* ids r, r + m, r + 2m, ... */
      const int32_t own = (s % m == r) ? (int32_t)(s / m) : -1;  /* s as a member number */
      draw_distinct_from(seed, OG_TAG_INIT, (uint32_t)s, 32 * r, 32, members, 0, own, draw);
      for (int j = 0; j < 32; ++j) {
        const int32_t id = draw[j] * m + r;
        row[32 * r + j].id = id;
        row[32 * r + j].d = og_distance(metric, d, vec, s, id);
        row[32 * r + j].isnew = 1;
        row[32 * r + j].fresh = 0;
      }
    }
    qsort(row, (size_t)k, sizeof(entry_t), entry_cmp);
    for (int j = 0; j < k; ++j) {
      ids[s * k + j] = row[j].id;
      dist[s * k + j] = row[j].d;
      isnew[s * k + j] = 1;
    }
  }
  free(row);
  free(draw);
}

/* ------------------------------------------------------------------------- */
/* ParallelSample (Alg. 1 line "G_old, G_new <- ParallelSample"; Sec. 4.1).
 *  1. forward: the first p NEW-flagged and the first p OLD-flagged entries of
 *     every list, in list order.  The sampled NEW entries become OLD now
 *     ("Mark all sampled neighbors as OLD", end of the loop body in Alg. 1: the
 *     join never reads flags, so clearing them here is equivalent).
 *  2. reverse: s is a candidate for the list of v for every forward sample v of
 *     s, per kind; candidates come from forward samples only ("derived from
 *     G_new itself").
 *  3. cap: the paper appends atomically until the list holds 2p entries and
 *     calls the outcome random sampling.  Reading: of the candidates of v keep
 *     the 2p - |forward(v)| with the smallest hash(seed, kind, v, s, iter)
 *     (upper 32 bits), ties by s - a random subset that does not depend on
 *     thread timing; all are kept when they fit.
 *  4. each list is sorted by id and duplicates removed.
 * Lists go to snew/sold (n rows of 2p ids, unused tail = -1), sizes to
 * cnew/cold. */
typedef struct {
  uint32_t key;
  int32_t s;
} revcand_t;

static int revcand_cmp(const void* pa, const void* pb) {
  const revcand_t* a = (const revcand_t*)pa;
  const revcand_t* b = (const revcand_t*)pb;
  if (a->key != b->key) return a->key < b->key ? -1 : 1;
  return (a->s > b->s) - (a->s < b->s);
}

static int int32_cmp(const void* pa, const void* pb) {
  int32_t a = *(const int32_t*)pa, b = *(const int32_t*)pb;
  return (a > b) - (a < b);
}

static void build_kind(int64_t n, int p, uint64_t seed, uint32_t tag, uint32_t iter,
                       const int32_t* fwd, const int32_t* nfwd, int32_t* out, int32_t* outcnt) {
  const int cap2p = 2 * p;
  int64_t* off = (int64_t*)calloc((size_t)n + 1, sizeof(int64_t));
  for (int64_t s = 0; s < n; ++s)
    for (int j = 0; j < nfwd[s]; ++j) off[fwd[s * p + j] + 1]++;
  for (int64_t v = 0; v < n; ++v) off[v + 1] += off[v];
  int64_t total = off[n];
  int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)(total ? total : 1));
  int64_t* cur = (int64_t*)malloc(sizeof(int64_t) * (size_t)n);
  memcpy(cur, off, sizeof(int64_t) * (size_t)n);
  for (int64_t s = 0; s < n; ++s)
    for (int j = 0; j < nfwd[s]; ++j) cand[cur[fwd[s * p + j]]++] = (int32_t)s;

  int64_t maxdeg = 1;
  for (int64_t v = 0; v < n; ++v)
    if (off[v + 1] - off[v] > maxdeg) maxdeg = off[v + 1] - off[v];
  revcand_t* rc = (revcand_t*)malloc(sizeof(revcand_t) * (size_t)maxdeg);
  int32_t* list = (int32_t*)malloc(sizeof(int32_t) * (size_t)cap2p);

  for (int64_t v = 0; v < n; ++v) {
    int64_t deg = off[v + 1] - off[v];
    for (int64_t e = 0; e < deg; ++e) {
      int32_t s = cand[off[v] + e];
      rc[e].s = s;
      rc[e].key = (uint32_t)(og_hash(seed, tag, (uint32_t)v, (uint32_t)s, iter) >> 32);
    }
    qsort(rc, (size_t)deg, sizeof(revcand_t), revcand_cmp);
    int m = 0;
    for (int j = 0; j < nfwd[v]; ++j) list[m++] = fwd[v * p + j];
    int room = cap2p - m;
    for (int64_t e = 0; e < deg && e < room; ++e) list[m++] = rc[e].s;
    qsort(list, (size_t)m, sizeof(int32_t), int32_cmp);
    int u = 0;
    for (int j = 0; j < m; ++j)
      if (j == 0 || list[j] != list[j - 1]) out[v * cap2p + u++] = list[j];
    outcnt[v] = u;
    for (int j = u; j < cap2p; ++j) out[v * cap2p + j] = -1;
  }
  free(off);
  free(cand);
  free(cur);
  free(rc);
  free(list);
}

void og_sample(int64_t n, int k, int p, uint64_t seed, uint32_t iter, const int32_t* ids,
               uint8_t* isnew, int32_t* snew, int32_t* cnew, int32_t* sold, int32_t* cold) {
  int32_t* fnew = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n * p));
  int32_t* fold = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n * p));
  int32_t* nfn = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  int32_t* nfo = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  for (int64_t s = 0; s < n; ++s) {
    int a = 0, b = 0;
    for (int j = 0; j < k; ++j) {
      int32_t v = ids[s * k + j];
      if (v < 0 || v >= n) continue; /* empty slot, or a frozen entry of a merge */
      if (isnew[s * k + j]) {
        if (a < p) {
          fnew[s * p + a++] = v;
          isnew[s * k + j] = 0;
        }
      } else if (b < p) {
        fold[s * p + b++] = v;
      }
    }
    nfn[s] = a;
    nfo[s] = b;
  }
  build_kind(n, p, seed, OG_TAG_REV_NEW, iter, fnew, nfn, snew, cnew);
  build_kind(n, p, seed, OG_TAG_REV_OLD, iter, fold, nfo, sold, cold);
  free(fnew);
  free(fold);
  free(nfn);
  free(nfo);
}

/* ------------------------------------------------------------------------- */
/* Eq. 1-2: the pair (u, v), v < u, that work item t of the NEW x NEW block
 * handles; its distance lives at slot u(u-1)/2 + v = t. */
void og_pair_of(int32_t t, int32_t* u, int32_t* v) {
  int32_t uu = (int32_t)ceil(sqrt(2.0 * (double)t + 2.25) - 0.5);
  *u = uu;
  *v = t - uu * (uu - 1) / 2;
}

/* Local join of one node with selective update (Alg. 1 inner loop; Sec. 4.2;
 * Sec. 4.3 "Selective update"; Alg. 2).
 * For node s with NEW samples N = snew[s] and OLD samples O = sold[s]:
 *   - distances of all unordered NEW pairs (triangular block, Eq. 1-2 order)
 *     and all NEW x OLD pairs (rectangular block);
 *   - for every NEW u: its nearest other NEW sample, and its nearest OLD
 *     sample; for every OLD u: its nearest NEW sample (Alg. 2 is a min
 *     reduction; ties by (distance, id)).
 * Each nearest object found becomes a proposal "insert v with distance d into
 * the list of u" (Alg. 1 InsertIntoNNList calls).
 * Readings: a pair whose two ids are equal (the same object sampled as NEW and
 * as OLD) is skipped and not counted.  Merge mode (split >= 0, Sec. 5.1 /
 * Alg. 3 comment): NEW x NEW distances are not calculated and a NEW x OLD pair
 * is evaluated only when its objects lie in different subsets (id < split vs
 * id >= split).
 * Output: up to 6p proposals per node in pu/pv/pd rows of 6p, count in pcnt;
 * returns the number of distances evaluated. */
uint64_t og_join(const void* vec, int64_t n, int d, int p, int metric, const int32_t* snew,
                 const int32_t* cnew, const int32_t* sold, const int32_t* cold, int64_t split,
                 int32_t* pu, int32_t* pv, double* pd, int32_t* pcnt) {
  const int L = 2 * p;
  uint64_t evals = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : evals)
  for (int64_t s = 0; s < n; ++s) {
    const int32_t* N = snew + s * L;
    const int32_t* O = sold + s * L;
    const int nn = cnew[s], no = cold[s];
    double* Dnn = (double*)malloc(sizeof(double) * (size_t)(L * (L - 1) / 2 + 1));
    double* Dno = (double*)malloc(sizeof(double) * (size_t)(L * L));
    uint8_t* Eno = (uint8_t*)malloc((size_t)(L * L)); /* pair evaluated? */
    const int do_nn = split < 0;
    if (do_nn) {
      for (int u = 1; u < nn; ++u)
        for (int v = 0; v < u; ++v) {
          Dnn[u * (u - 1) / 2 + v] = og_distance(metric, d, vec, N[u], N[v]);
          ++evals;
        }
    }
    for (int a = 0; a < nn; ++a)
      for (int b = 0; b < no; ++b) {
        int ok = N[a] != O[b];
        if (ok && split >= 0) ok = ((N[a] < split) != (O[b] < split));
        Eno[a * L + b] = (uint8_t)ok;
        if (ok) {
          Dno[a * L + b] = og_distance(metric, d, vec, N[a], O[b]);
          ++evals;
        }
      }
    int m = 0;
    int32_t* qu = pu + s * 3 * L;
    int32_t* qv = pv + s * 3 * L;
    double* qd = pd + s * 3 * L;
    for (int a = 0; a < nn; ++a) {
      /* nearest other NEW sample of N[a] */
      if (do_nn) {
        int best = -1;
        double bd = 0;
        for (int c = 0; c < nn; ++c) {
          if (c == a) continue;
          int hi = a > c ? a : c, lo = a > c ? c : a;
          double dist = Dnn[hi * (hi - 1) / 2 + lo];
          if (best < 0 || closer(dist, N[c], bd, N[best])) {
            best = c;
            bd = dist;
          }
        }
        if (best >= 0) {
          qu[m] = N[a];
          qv[m] = N[best];
          qd[m] = bd;
          ++m;
        }
      }
      /* nearest OLD sample of N[a] */
      int best = -1;
      double bd = 0;
      for (int b = 0; b < no; ++b) {
        if (!Eno[a * L + b]) continue;
        double dist = Dno[a * L + b];
        if (best < 0 || closer(dist, O[b], bd, O[best])) {
          best = b;
          bd = dist;
        }
      }
      if (best >= 0) {
        qu[m] = N[a];
        qv[m] = O[best];
        qd[m] = bd;
        ++m;
      }
    }
    for (int b = 0; b < no; ++b) {
      /* nearest NEW sample of O[b] */
      int best = -1;
      double bd = 0;
      for (int a = 0; a < nn; ++a) {
        if (!Eno[a * L + b]) continue;
        double dist = Dno[a * L + b];
        if (best < 0 || closer(dist, N[a], bd, N[best])) {
          best = a;
          bd = dist;
        }
      }
      if (best >= 0) {
        qu[m] = O[b];
        qv[m] = N[best];
        qd[m] = bd;
        ++m;
      }
    }
    pcnt[s] = m;
    free(Dnn);
    free(Dno);
    free(Eno);
  }
  return evals;
}

/* The join without the selective update of Sec. 4.3 (the variant the ablation of
 * Sec. 6.2 calls GNND-r1): the same pairs are evaluated, and every evaluated
 * pair (a, b) is proposed both ways, b for the list of a and a for the list of
 * b.  Output rows of 2p(6p - 1) slots per node: NEW x NEW gives nn(nn - 1)
 * proposals, NEW x OLD 2 nn no, with nn, no <= 2p.  Returns the number of
 * distances evaluated. */
uint64_t og_join_all(const void* vec, int64_t n, int d, int p, int metric, const int32_t* snew,
                     const int32_t* cnew, const int32_t* sold, const int32_t* cold, int64_t split,
                     int32_t* pu, int32_t* pv, double* pd, int32_t* pcnt) {
  const int L = 2 * p;
  const int64_t P = (int64_t)L * (3 * L - 1);
  uint64_t evals = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : evals)
  for (int64_t s = 0; s < n; ++s) {
    const int32_t* N = snew + s * L;
    const int32_t* O = sold + s * L;
    const int nn = cnew[s], no = cold[s];
    int32_t* qu = pu + s * P;
    int32_t* qv = pv + s * P;
    double* qd = pd + s * P;
    int m = 0;
    if (split < 0) {
      for (int a = 1; a < nn; ++a)
        for (int b = 0; b < a; ++b) {
          const double dist = og_distance(metric, d, vec, N[a], N[b]);
          ++evals;
          qu[m] = N[a]; qv[m] = N[b]; qd[m] = dist; ++m;
          qu[m] = N[b]; qv[m] = N[a]; qd[m] = dist; ++m;
        }
    }
    for (int a = 0; a < nn; ++a)
      for (int b = 0; b < no; ++b) {
        if (N[a] == O[b]) continue;
        if (split >= 0 && ((N[a] < split) == (O[b] < split))) continue;
        const double dist = og_distance(metric, d, vec, N[a], O[b]);
        ++evals;
        qu[m] = N[a]; qv[m] = O[b]; qd[m] = dist; ++m;
        qu[m] = O[b]; qv[m] = N[a]; qd[m] = dist; ++m;
      }
    pcnt[s] = m;
  }
  return evals;
}

/* ------------------------------------------------------------------------- */
/* InsertIntoNNList for one (v, d) into one sorted list of k entries
 * (Sec. 4.3): refused when v is already present or when (d, v) is not closer
 * than the last entry; otherwise the entry takes its sorted place, the tail
 * shifts by one, the last entry drops out, and the new entry is flagged NEW.
 * Returns 1 when inserted.  (Used to show that the order of insertions does
 * not matter; og_update below is the whole-iteration form.) */
int og_insert_one(int k, int32_t* ids, double* dist, uint8_t* isnew, int32_t v, double d) {
  for (int j = 0; j < k; ++j)
    if (ids[j] == v) return 0;
  if (!closer(d, v, dist[k - 1], ids[k - 1])) return 0;
  int pos = k - 1;
  while (pos > 0 && closer(d, v, dist[pos - 1], ids[pos - 1])) {
    ids[pos] = ids[pos - 1];
    dist[pos] = dist[pos - 1];
    isnew[pos] = isnew[pos - 1];
    --pos;
  }
  ids[pos] = v;
  dist[pos] = d;
  isnew[pos] = 1;
  return 1;
}

/* The local join of classic NN-Descent (Sec. 3, the CPU scheme the paper starts
 * from), for comparison only: node after node, every NEW x NEW and NEW x OLD
 * pair of the node's sample lists is evaluated and tried at once on both
 * lists (og_insert_one), so later joins of the same iteration see the lists
 * as earlier ones left them.  Sequential by definition.  Returns the number
 * of distances evaluated; *inserts counts the accepted insertions. */
uint64_t og_classic_join_update(const void* vec, int64_t n, int d, int k, int p, int metric,
                                const int32_t* snew, const int32_t* cnew, const int32_t* sold,
                                const int32_t* cold, int32_t* ids, double* dist, uint8_t* isnew,
                                uint64_t* inserts) {
  const int L = 2 * p;
  uint64_t evals = 0, ins = 0;
  for (int64_t s = 0; s < n; ++s) {
    const int32_t* N = snew + s * L;
    const int32_t* O = sold + s * L;
    const int nn = cnew[s], no = cold[s];
    for (int a = 0; a < nn; ++a) {
      for (int b = 0; b < a; ++b) {
        const double dd = og_distance(metric, d, vec, N[a], N[b]);
        ++evals;
        ins += (uint64_t)og_insert_one(k, ids + (int64_t)N[a] * k, dist + (int64_t)N[a] * k,
                                       isnew + (int64_t)N[a] * k, N[b], dd);
        ins += (uint64_t)og_insert_one(k, ids + (int64_t)N[b] * k, dist + (int64_t)N[b] * k,
                                       isnew + (int64_t)N[b] * k, N[a], dd);
      }
      for (int b = 0; b < no; ++b) {
        if (N[a] == O[b]) continue;
        const double dd = og_distance(metric, d, vec, N[a], O[b]);
        ++evals;
        ins += (uint64_t)og_insert_one(k, ids + (int64_t)N[a] * k, dist + (int64_t)N[a] * k,
                                       isnew + (int64_t)N[a] * k, O[b], dd);
        ins += (uint64_t)og_insert_one(k, ids + (int64_t)O[b] * k, dist + (int64_t)O[b] * k,
                                       isnew + (int64_t)O[b] * k, N[a], dd);
      }
    }
  }
  *inserts = ins;
  return evals;
}

/* Graph update of one iteration (all InsertIntoNNList calls of Alg. 1).
 * The paper inserts concurrently under (segment) spinlocks.  Reading: the list
 * of u after the iteration is the first k, by (distance, id), of its entries
 * before the iteration united with all proposals made for u, one entry per id -
 * the outcome of the insertions in any order.  Entries that stay keep their
 * flag; admitted ones are NEW (Sec. 4, "newly inserted ... marked as NEW").
 * Returns the number of admitted entries (list members that were not members
 * before). */
uint64_t og_update_rows(int64_t n, int k, int P, int32_t* ids, double* dist, uint8_t* isnew,
                        const int32_t* pu, const int32_t* pv, const double* pd,
                        const int32_t* pcnt);
static uint64_t update_classes(int64_t n, int k, int P, int classes, int32_t* ids, double* dist,
                               uint8_t* isnew, const int32_t* pu, const int32_t* pv,
                               const double* pd, const int32_t* pcnt);
uint64_t og_update(int64_t n, int k, int p, int32_t* ids, double* dist, uint8_t* isnew,
                   const int32_t* pu, const int32_t* pv, const double* pd, const int32_t* pcnt) {
  return og_update_rows(n, k, 6 * p, ids, dist, isnew, pu, pv, pd, pcnt);
}
/* The same with proposal rows of P slots per joined node. */
uint64_t og_update_rows(int64_t n, int k, int P, int32_t* ids, double* dist, uint8_t* isnew,
                        const int32_t* pu, const int32_t* pv, const double* pd,
                        const int32_t* pcnt) {
  return update_classes(n, k, P, 1, ids, dist, isnew, pu, pv, pd, pcnt);
}
/* Insertion into segmented lists (Sec. 4.3, "Multiple Spinlocks"): "the object v will be
 * inserted into the v % (k / 32)-th segment", each segment "keeps 32 neighbors", and "as the
 * iteration is completed, all the segments of one k-NN list will be merged into one".  As a
 * set function: per residue class of the ids (m = k / 32 classes) the 32 best, by
 * (distance, id), of the class's entries before the iteration and the proposals of that
 * class, one entry per id; the list is their union, ascending.  m = 1 is the plain list. */
uint64_t og_update_segmented(int64_t n, int k, int P, int32_t* ids, double* dist, uint8_t* isnew,
                             const int32_t* pu, const int32_t* pv, const double* pd,
                             const int32_t* pcnt) {
  return update_classes(n, k, P, k / 32, ids, dist, isnew, pu, pv, pd, pcnt);
}
/* `classes` classes of ids (v % classes), each holding at most k / classes entries. */
static uint64_t update_classes(int64_t n, int k, int P, int classes, int32_t* ids, double* dist,
                               uint8_t* isnew, const int32_t* pu, const int32_t* pv,
                               const double* pd, const int32_t* pcnt) {
  int64_t* off = (int64_t*)calloc((size_t)n + 1, sizeof(int64_t));
  for (int64_t s = 0; s < n; ++s)
    for (int j = 0; j < pcnt[s]; ++j) off[pu[s * P + j] + 1]++;
  for (int64_t u = 0; u < n; ++u) off[u + 1] += off[u];
  int64_t total = off[n];
  int32_t* bv = (int32_t*)malloc(sizeof(int32_t) * (size_t)(total ? total : 1));
  double* bd = (double*)malloc(sizeof(double) * (size_t)(total ? total : 1));
  int64_t* cur = (int64_t*)malloc(sizeof(int64_t) * (size_t)n);
  memcpy(cur, off, sizeof(int64_t) * (size_t)n);
  int64_t maxm = 0;
  for (int64_t s = 0; s < n; ++s)
    for (int j = 0; j < pcnt[s]; ++j) {
      int32_t u = pu[s * P + j];
      bv[cur[u]] = pv[s * P + j];
      bd[cur[u]] = pd[s * P + j];
      cur[u]++;
    }
  for (int64_t u = 0; u < n; ++u)
    if (off[u + 1] - off[u] > maxm) maxm = off[u + 1] - off[u];
  entry_t* pool = (entry_t*)malloc(sizeof(entry_t) * (size_t)(maxm + k));
  uint64_t inserts = 0;
  for (int64_t u = 0; u < n; ++u) {
    int64_t m = 0;
    for (int j = 0; j < k; ++j) {
      if (ids[u * k + j] < 0) continue;
      pool[m].id = ids[u * k + j];
      pool[m].d = dist[u * k + j];
      pool[m].isnew = isnew[u * k + j];
      pool[m].fresh = 0;
      ++m;
    }
    for (int64_t e = off[u]; e < off[u + 1]; ++e) {
      pool[m].id = bv[e];
      pool[m].d = bd[e];
      pool[m].isnew = 1;
      pool[m].fresh = 1;
      ++m;
    }
    qsort(pool, (size_t)m, sizeof(entry_t), entry_cmp);
    int w = 0;
    int held[4] = {0, 0, 0, 0};  /* entries taken per class (at most 4 classes: k <= 128) */
    for (int64_t e = 0; e < m && w < k; ++e) {
      int dup = 0;
      for (int j = 0; j < w && !dup; ++j) dup = (ids[u * k + j] == pool[e].id);
      if (dup) continue;
      if (held[pool[e].id % classes] >= k / classes) continue;  /* its segment is full */
      held[pool[e].id % classes]++;
      ids[u * k + w] = pool[e].id;
      dist[u * k + w] = pool[e].d;
      isnew[u * k + w] = pool[e].isnew;
      inserts += pool[e].fresh;
      ++w;
    }
    for (; w < k; ++w) {
      ids[u * k + w] = -1;
      dist[u * k + w] = INFINITY;
      isnew[u * k + w] = 0;
    }
  }
  free(off);
  free(bv);
  free(bd);
  free(cur);
  free(pool);
  return inserts;
}

/* ------------------------------------------------------------------------- */
/* Numbering inside one merge.  The two sets occupy the id ranges
 * [base1, base1 + n1) and [base2, base2 + n2) of a larger collection (the
 * shards of Sec. 5.1).  Inside the merge the objects of S1 are numbered
 * 0..n1-1 and those of S2 n1..n-1 (n = n1 + n2); any other object - a list
 * entry that came from an earlier merge with a third shard - is numbered
 * n + its collection id.  Reading (the paper is silent on such entries): they
 * are frozen - they keep their place in the list by their stored distance and
 * compete with every insertion, but they are never sampled and so never take
 * part in a join, because their vectors are not there. */
int32_t og_to_internal(int64_t g, int64_t n1, int64_t base1, int64_t n2, int64_t base2) {
  if (g >= base1 && g < base1 + n1) return (int32_t)(g - base1);
  if (g >= base2 && g < base2 + n2) return (int32_t)(n1 + g - base2);
  return (int32_t)(n1 + n2 + g);
}

int32_t og_to_global(int64_t i, int64_t n1, int64_t base1, int64_t n2, int64_t base2) {
  if (i < n1) return (int32_t)(base1 + i);
  if (i < n1 + n2) return (int32_t)(base2 + i - n1);
  return (int32_t)(i - n1 - n2);
}

/* GGM initialisation (Alg. 3, "Divide" and "Append" steps; Sec. 5.1).
 * The merged graph has n1 + n2 lists, S1's nodes first; the input lists carry
 * collection ids, which are renumbered as above.
 * Every list keeps its first ceil(k/2) entries, flagged OLD; the other
 * floor(k/2) entries are set aside (aside_*: n rows of floor(k/2)) and replaced
 * by floor(k/2) distinct random objects of the other subset with their
 * distances, flagged NEW.  Reading: the refilled list is put back into
 * (distance, id) order, because sampling takes "the first p" of a sorted list.
 * Requires min(n1, n2) >= floor(k/2). */
void og_merge_init(const void* vec, int64_t n1, int64_t base1, int64_t n2, int64_t base2, int d,
                   int k, int metric, uint64_t seed, const int32_t* ids1, const double* dist1,
                   const int32_t* ids2, const double* dist2, int32_t* ids, double* dist,
                   uint8_t* isnew, int32_t* aside_ids, double* aside_dist) {
  const int keep = (k + 1) / 2, fill = k / 2;
  const int64_t n = n1 + n2;
  entry_t* row = (entry_t*)malloc(sizeof(entry_t) * (size_t)k);
  int32_t* draw = (int32_t*)malloc(sizeof(int32_t) * (size_t)(fill ? fill : 1));
  for (int64_t s = 0; s < n; ++s) {
    const int first = s < n1;
    const int32_t* sid = first ? ids1 + s * k : ids2 + (s - n1) * k;
    const double* sdist = first ? dist1 + s * k : dist2 + (s - n1) * k;
    for (int j = 0; j < keep; ++j) {
      row[j].id = og_to_internal(sid[j], n1, base1, n2, base2);
      row[j].d = sdist[j];
      row[j].isnew = 0;
      row[j].fresh = 0;
    }
    for (int j = 0; j < fill; ++j) {
      aside_ids[s * fill + j] = og_to_internal(sid[keep + j], n1, base1, n2, base2);
      aside_dist[s * fill + j] = sdist[keep + j];
    }
    draw_distinct(seed, OG_TAG_MERGE, (uint32_t)s, fill, (uint32_t)(first ? n2 : n1),
                  first ? (int32_t)n1 : 0, -1, draw);
    for (int j = 0; j < fill; ++j) {
      row[keep + j].id = draw[j];
      row[keep + j].d = og_distance(metric, d, vec, s, draw[j]);
      row[keep + j].isnew = 1;
      row[keep + j].fresh = 0;
    }
    qsort(row, (size_t)k, sizeof(entry_t), entry_cmp);
    for (int j = 0; j < k; ++j) {
      ids[s * k + j] = row[j].id;
      dist[s * k + j] = row[j].d;
      isnew[s * k + j] = row[j].isnew;
    }
  }
  free(row);
  free(draw);
}

/* GGM last step ("Merge and Sort G with G1^v and G2^v", Alg. 3): per node the
 * first k by (distance, id) of the refined list united with its set-aside
 * half, one entry per id. */
void og_merge_final(int64_t n, int k, int32_t* ids, double* dist, const int32_t* aside_ids,
                    const double* aside_dist) {
  const int fill = k / 2;
  entry_t* pool = (entry_t*)malloc(sizeof(entry_t) * (size_t)(k + fill));
  for (int64_t s = 0; s < n; ++s) {
    int m = 0;
    for (int j = 0; j < k; ++j) {
      pool[m].id = ids[s * k + j];
      pool[m].d = dist[s * k + j];
      pool[m].isnew = 0;
      pool[m].fresh = 0;
      ++m;
    }
    for (int j = 0; j < fill; ++j) {
      pool[m].id = aside_ids[s * fill + j];
      pool[m].d = aside_dist[s * fill + j];
      pool[m].isnew = 0;
      pool[m].fresh = 1;
      ++m;
    }
    qsort(pool, (size_t)m, sizeof(entry_t), entry_cmp);
    int w = 0;
    for (int e = 0; e < m && w < k; ++e) {
      int dup = 0;
      for (int j = 0; j < w && !dup; ++j) dup = (ids[s * k + j] == pool[e].id);
      if (dup) continue;
      ids[s * k + w] = pool[e].id;
      dist[s * k + w] = pool[e].d;
      ++w;
    }
  }
  free(pool);
}

/* Back to collection ids after a merge: renumber every entry and restore the
 * (distance, id) order of each list under the collection ids. */
void og_merge_to_global(int64_t n1, int64_t base1, int64_t n2, int64_t base2, int k,
                        int32_t* ids, double* dist) {
  entry_t* row = (entry_t*)malloc(sizeof(entry_t) * (size_t)k);
  for (int64_t s = 0; s < n1 + n2; ++s) {
    for (int j = 0; j < k; ++j) {
      row[j].id = og_to_global(ids[s * k + j], n1, base1, n2, base2);
      row[j].d = dist[s * k + j];
      row[j].isnew = 0;
      row[j].fresh = 0;
    }
    qsort(row, (size_t)k, sizeof(entry_t), entry_cmp);
    for (int j = 0; j < k; ++j) {
      ids[s * k + j] = row[j].id;
      dist[s * k + j] = row[j].d;
    }
  }
  free(row);
}
