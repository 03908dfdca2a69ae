/*
 * CPU oracle for the block-based inverted-list index (arXiv 2408.02937).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, sequential statement of
 * what the index computes, written from the paper; it shares no code with the
 * HIP library and must never be on the product path.  Only the tests, the
 * smoke check and the benchmark's CPU-baseline leg may load it.
 *
 * What follows which passage of the paper:
 *   orc_assign      Insertion algorithm, the step "k <- min(c, y_i) for all c":
 *                   nearest centroid of a new vector.
 *   orc_add         Insertion algorithm, the loop over new vectors: take the
 *                   next position did of list k, mid = did / T_m,
 *                   moff = did % T_m, open a new block from the pool when
 *                   mid is past the chain's end (only ever with moff == 0),
 *                   then the Exceed() test (the equation defining Exceed) and
 *                   the call to Rearrangement.
 *   orc_rearrange   Rearrangement algorithm and the sentence introducing it:
 *                   the physical neighbour of the chain's first block is
 *                   exchanged with the next linked block of the chain, so the
 *                   chain becomes contiguous and header jumps disappear.
 *   orc_search      Introduction, description of inverted-index search: the
 *                   lists of the clusters most relevant to the query are
 *                   scanned and the top-k of them is returned.  Distances are
 *                   exact (IVF-Flat), so this is the textbook definition.
 *
 * Readings where the paper is silent (each one also listed in the design
 * notes of this repository):
 *   - "min(c, y)" is the squared Euclidean distance for the L2 metric and the
 *     (negated) inner product for the IP metric; ties go to the lowest index.
 *   - The coarse score that DECIDES an integer (which list, which probes) is
 *     computed in one fixed arithmetic so that two implementations can agree
 *     bit for bit: IEEE double, one fused multiply-add per dimension, in
 *     dimension order 0..d-1.
 *   - The fine score is the plain definition in double: sum_j (x_j-q_j)^2 or
 *     sum_j x_j*q_j, accumulated in dimension order with separate multiply
 *     and add.  L2 is returned squared.
 *   - Results are ordered by (score, id): ascending score for L2, descending
 *     score for IP, ascending id among equal scores.  Missing results are
 *     id -1 with +inf (L2) or -inf (IP).
 *   - ids are the caller's, or ntotal + i when none are given (the running
 *     total "gid" of the Insertion algorithm).
 *   - Exceed() counts the vectors appended to the list since its last
 *     rearrangement and is a strict ">".
 *
 * Product-quantised lists (the paper names IVF-PQ beside IVF-Flat as an index
 * kind whose lists live in the same blocks, without spelling it out; this is
 * the textbook method, J\'egou et al. 2011, with these readings):
 *   - the codebooks are given (training is outside the path): M sub-spaces of
 *     d / M dimensions, 256 entries each;
 *   - a vector is coded as it is (not its residual to the coarse centroid), so
 *     one table of sub-distances per query serves all lists;
 *   - code m of a vector is the entry of codebook m nearest to sub-vector m in
 *     squared Euclidean distance (for both metrics), computed in the fixed
 *     arithmetic (double, one fma per dimension, in order), ties to the lowest
 *     entry: codes are integers both implementations must agree on;
 *   - the score of a coded vector is the sum over m, in order, of the table
 *     entry of its code: squared distance (L2) or inner product (IP) between
 *     the query's sub-vector and the codebook entry, plain double arithmetic.
 *   orc_set_codebooks / orc_pq_encode / orc_add / orc_search follow that.
 *
 * Narrow storage of flat lists (a step towards the quantised lists that keeps
 * the vectors themselves; the paper stores 32-bit floats): a list may hold its
 * vectors as IEEE half-precision numbers or as bytes.  Readings:
 *   - a vector joins the list of its nearest centroid as it is given; what the
 *     list keeps, returns and scans is the vector after the conversion;
 *   - half: round to nearest, ties to even, values past the largest half
 *     become infinity (the IEEE conversion);
 *   - byte: rounded to the nearest integer, ties to even, then clamped to
 *     0..255; not-a-number becomes 0.  (Byte-valued data is kept exactly.)
 *   - scores are computed as for 32-bit storage, on the converted vectors.
 *   orc_set_storage / orc_stored follow that.
 *
 * Pins (tests/test_oracle_*.py): brute-force exact k-NN when every list is
 * probed; restriction to the probed lists otherwise; ranking by the double
 * scores where their float roundings coincide; membership invariants; closed
 * forms for block counts and slot addresses; the pad-memory figure of the
 * block-size experiment; rearrangement scenarios worked by hand (the figure-1
 * style exchange, a rearranged list as the next victim, a target on the free
 * stack of a full pool, the end of the pool); the strictness of Exceed();
 * numpy's IEEE conversions and brute force over independently converted
 * vectors for the narrow storage; exact-rational emulation of the coarse
 * arithmetic.  (Each was seen to fail when the matching mistake was planted in
 * a copy of this file.)
 * Parity unpinned: the order of vectors of one batch inside a list and the
 * physical block numbers (several results are correct; compared canonically).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_L2 = 0, ORC_IP = 1 };
enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_ESTATE = -2, ORC_EPOOL = -3 };
enum { ORC_F32 = 0, ORC_F16 = 1, ORC_U8 = 2 };

typedef struct {
  int64_t n, cap;      /* logical length and capacity of the arrays below   */
  int64_t *ids;        /* [n]                                                */
  float *x;            /* [n][d] row-major (flat lists)                      */
  uint8_t *codes;      /* [n][M] (product-quantised lists)                   */
  int64_t online;      /* vectors appended since the last rearrangement      */
  int32_t *chain;      /* physical block numbers, in logical order           */
  int64_t nchain, chain_cap;
} orc_list;

typedef struct {
  int d, nlist, metric;
  int64_t T_m;         /* block capacity in vectors                          */
  int64_t T_mp;        /* rearrangement threshold in vectors, <= 0: never    */
  float *C;            /* [nlist][d]                                         */
  int has_C;
  int pq_m;            /* sub-spaces of a product quantiser, 0: flat lists    */
  float *CB;           /* [M][256][d / M] codebooks                          */
  int storage;         /* ORC_F32 / ORC_F16 / ORC_U8: what flat lists keep     */
  orc_list *L;
  int64_t npool;       /* |P|: number of blocks in the central pool          */
  int64_t cur_P;       /* blocks 0..cur_P-1 have been handed out at least once */
  int32_t *free_blocks;/* stack of returned blocks                           */
  int64_t nfree;
  int32_t *owner;      /* per physical block: owning list or -1              */
  int32_t *seq;        /* per physical block: position in the owner's chain  */
  int64_t ntotal;
  int64_t n_rearrange; /* how many times Rearrangement ran                   */
} orc_index;

/* ---------------------------------------------------------------- helpers */

static int better(int metric, double a, double b) {
  /* is score a strictly better than score b? */
  return metric == ORC_L2 ? (a < b) : (a > b);
}

/* Coarse score in the fixed arithmetic: one fma per dimension, in order. */
static double coarse_score(int metric, int d, const float *y, const float *c) {
  double acc = 0.0;
  if (metric == ORC_L2) {
    for (int j = 0; j < d; ++j) {
      double t = (double)y[j] - (double)c[j];
      acc = fma(t, t, acc);
    }
  } else {
    for (int j = 0; j < d; ++j) acc = fma((double)y[j], (double)c[j], acc);
  }
  return acc;
}

/* Fine score: the plain definition in double. */
static double fine_score(int metric, int d, const float *x, const float *q) {
  double acc = 0.0;
  if (metric == ORC_L2) {
    for (int j = 0; j < d; ++j) {
      double t = (double)x[j] - (double)q[j];
      acc = acc + t * t;
    }
  } else {
    for (int j = 0; j < d; ++j) acc = acc + (double)x[j] * (double)q[j];
  }
  return acc;
}

static int nearest_centroid(const orc_index *ix, const float *y) {
  int best = 0;
  double bs = coarse_score(ix->metric, ix->d, y, ix->C);
  for (int c = 1; c < ix->nlist; ++c) {
    double s = coarse_score(ix->metric, ix->d, y, ix->C + (size_t)c * ix->d);
    if (better(ix->metric, s, bs)) { bs = s; best = c; }
  }
  return best;
}

/* ------------------------------------------------------------- life cycle */

orc_index *orc_create(int d, int nlist, int metric, int64_t T_m, int64_t T_mp, int64_t npool) {
  if (d <= 0 || nlist <= 0 || T_m <= 0 || npool < 0 || (metric != ORC_L2 && metric != ORC_IP))
    return NULL;
  orc_index *ix = (orc_index *)calloc(1, sizeof(orc_index));
  ix->d = d; ix->nlist = nlist; ix->metric = metric; ix->T_m = T_m; ix->T_mp = T_mp;
  ix->C = (float *)calloc((size_t)nlist * d, sizeof(float));
  ix->L = (orc_list *)calloc((size_t)nlist, sizeof(orc_list));
  ix->npool = npool;
  ix->free_blocks = (int32_t *)calloc((size_t)npool + 1, sizeof(int32_t));
  ix->owner = (int32_t *)malloc(((size_t)npool + 1) * sizeof(int32_t));
  ix->seq = (int32_t *)calloc((size_t)npool + 1, sizeof(int32_t));
  for (int64_t b = 0; b < npool; ++b) ix->owner[b] = -1;
  return ix;
}

void orc_destroy(orc_index *ix) {
  if (!ix) return;
  for (int k = 0; k < ix->nlist; ++k) {
    free(ix->L[k].ids); free(ix->L[k].x); free(ix->L[k].codes); free(ix->L[k].chain);
  }
  free(ix->CB);
  free(ix->L); free(ix->C); free(ix->free_blocks); free(ix->owner); free(ix->seq); free(ix);
}

int orc_set_centroids(orc_index *ix, const float *C) {
  if (!ix || !C) return ORC_EINVAL;
  memcpy(ix->C, C, (size_t)ix->nlist * ix->d * sizeof(float));
  ix->has_C = 1;
  return ORC_OK;
}

/* What a flat list keeps of a coordinate.  Half precision: the number is
 * rounded to a multiple of the spacing of halves at its magnitude, 2^(e-10)
 * for a number in [2^e, 2^(e+1)) and 2^-24 below 2^-14 (subnormal halves);
 * rintf rounds to nearest, ties to even, and the scalings by powers of two are
 * exact.  The largest half is 65504. */
static float stored_value(int storage, float f) {
  if (storage == ORC_F16) {
    if (isnan(f) || isinf(f) || f == 0.0f) return f;
    int e;
    (void)frexpf(fabsf(f), &e);           /* |f| = m 2^e with m in [0.5, 1) */
    int q = e - 11;                       /* exponent of the spacing */
    if (q < -24) q = -24;
    float r = ldexpf(rintf(ldexpf(f, -q)), q);
    if (fabsf(r) > 65504.0f) r = copysignf(INFINITY, f);
    return r;
  }
  if (storage == ORC_U8) {
    if (isnan(f)) return 0.0f;
    float r = rintf(f);
    return r > 0.0f ? (r > 255.0f ? 255.0f : r) : 0.0f;
  }
  return f;
}

/* Storage of flat lists; only before the first vector is added. */
int orc_set_storage(orc_index *ix, int storage) {
  if (!ix || storage < ORC_F32 || storage > ORC_U8) return ORC_EINVAL;
  if (ix->ntotal > 0 || ix->pq_m) return ORC_ESTATE;
  ix->storage = storage;
  return ORC_OK;
}

/* The conversion by itself: out[i] = what a list with this storage keeps of in[i]. */
void orc_stored(int storage, int64_t n, const float *in, float *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = stored_value(storage, in[i]);
}

/* Codebooks of a product quantiser: CB [M][256][d / M].  Only before the
 * first vector is added. */
int orc_set_codebooks(orc_index *ix, int M, const float *CB) {
  if (!ix || !CB || M < 1 || ix->d % M != 0) return ORC_EINVAL;
  if (ix->ntotal > 0 || ix->storage != ORC_F32) return ORC_ESTATE;
  free(ix->CB);
  ix->CB = (float *)malloc((size_t)256 * ix->d * sizeof(float));
  memcpy(ix->CB, CB, (size_t)256 * ix->d * sizeof(float));
  ix->pq_m = M;
  return ORC_OK;
}

/* Code of sub-vector m: nearest codebook entry, fixed arithmetic, ties low. */
static uint8_t pq_code(const orc_index *ix, int m, const float *ysub) {
  const int ds = ix->d / ix->pq_m;
  const float *cb = ix->CB + (size_t)m * 256 * ds;
  int best = 0;
  double bs = coarse_score(ORC_L2, ds, ysub, cb);
  for (int c = 1; c < 256; ++c) {
    double s = coarse_score(ORC_L2, ds, ysub, cb + (size_t)c * ds);
    if (s < bs) { bs = s; best = c; }
  }
  return (uint8_t)best;
}

/* Codes of n vectors: out [n][M]. */
int orc_pq_encode(const orc_index *ix, int64_t n, const float *Y, uint8_t *out) {
  if (!ix || ix->pq_m == 0) return ORC_ESTATE;
  const int M = ix->pq_m, ds = ix->d / M;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i)
    for (int m = 0; m < M; ++m)
      out[(size_t)i * M + m] = pq_code(ix, m, Y + (size_t)i * ix->d + (size_t)m * ds);
  return ORC_OK;
}

/* ------------------------------------------------------------- assignment */

/* Nearest centroid of each of n vectors.  Independent per vector, so the loop
 * may run on several cores; the result does not depend on that. */
int orc_assign(const orc_index *ix, int64_t n, const float *Y, int32_t *out) {
  if (!ix || !ix->has_C) return ORC_ESTATE;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = nearest_centroid(ix, Y + (size_t)i * ix->d);
  return ORC_OK;
}

/* Coarse scores of one vector against every centroid (out [nlist] double), in
 * the fixed arithmetic.  Exposed so a test can check the arithmetic itself. */
int orc_coarse_scores(const orc_index *ix, const float *y, double *out) {
  if (!ix || !ix->has_C) return ORC_ESTATE;
  for (int c = 0; c < ix->nlist; ++c)
    out[c] = coarse_score(ix->metric, ix->d, y, ix->C + (size_t)c * ix->d);
  return ORC_OK;
}

/* ------------------------------------------------------------ block model */

static int take_block(orc_index *ix, int32_t *out) {
  if (ix->nfree > 0) { *out = ix->free_blocks[--ix->nfree]; return ORC_OK; }
  if (ix->cur_P >= ix->npool) return ORC_EPOOL;
  *out = (int32_t)ix->cur_P++;   /* the atomicAdd(cur_P, 1) of the paper, done serially */
  return ORC_OK;
}

static void give_block(orc_index *ix, int32_t b) {
  ix->owner[b] = -1;
  ix->free_blocks[ix->nfree++] = b;
}

static void unfree_block(orc_index *ix, int32_t b) {
  for (int64_t i = 0; i < ix->nfree; ++i)
    if (ix->free_blocks[i] == b) {
      ix->free_blocks[i] = ix->free_blocks[--ix->nfree];
      return;
    }
}

/* Rearrangement of list k.  Target: block t of the chain sits at physical
 * position b0 + t, where b0 is the chain's first block.  Walk the chain; when
 * the next linked block is not the physical neighbour, exchange the two
 * blocks' contents and owners (a plain move when the neighbour holds nothing).
 * The victim list keeps its logical content but its chain now points at the
 * block the target list gave up. */
int orc_rearrange(orc_index *ix, int k) {
  if (!ix || k < 0 || k >= ix->nlist) return ORC_EINVAL;
  orc_list *l = &ix->L[k];
  ix->n_rearrange++;
  l->online = 0;
  if (l->nchain <= 1) return ORC_OK;
  int64_t b0 = l->chain[0];
  for (int64_t t = 1; t < l->nchain; ++t) {
    int64_t tgt = b0 + t;
    int32_t src = l->chain[t];
    if (tgt >= ix->npool) break;        /* the pool ends here: stay partly compacted */
    if (src == tgt) continue;
    int occupied = 0;
    if (tgt >= ix->cur_P) {             /* never handed out (targets advance one block at a
                                           time, so tgt == cur_P): the frontier moves past it */
      ix->cur_P = tgt + 1;
    } else if (ix->owner[tgt] < 0) {    /* sits on the free stack */
      unfree_block(ix, (int32_t)tgt);
    } else {
      occupied = 1;
    }
    if (occupied) {
      int32_t v = ix->owner[tgt], s = ix->seq[tgt];
      ix->L[v].chain[s] = src;          /* victim (may be list k itself, further down) */
      ix->owner[src] = v; ix->seq[src] = s;
    } else {
      give_block(ix, src);
    }
    ix->owner[tgt] = k; ix->seq[tgt] = (int32_t)t;
    l->chain[t] = (int32_t)tgt;
  }
  return ORC_OK;
}

/* ---------------------------------------------------------------- insertion */

static void list_reserve(orc_list *l, int d, int pq_m, int64_t need) {
  if (need <= l->cap) return;
  int64_t cap = l->cap ? l->cap : 16;
  while (cap < need) cap *= 2;
  l->ids = (int64_t *)realloc(l->ids, (size_t)cap * sizeof(int64_t));
  if (pq_m) l->codes = (uint8_t *)realloc(l->codes, (size_t)cap * pq_m);
  else l->x = (float *)realloc(l->x, (size_t)cap * d * sizeof(float));
  l->cap = cap;
}

/* Insert n vectors, one after the other in input order.  `assign` may carry
 * the lists computed by orc_assign (to reuse a parallel pass); NULL computes
 * them here.  Returns ORC_EPOOL, with nothing inserted, when the pool cannot
 * hold the blocks this batch needs. */
int orc_add(orc_index *ix, int64_t n, const float *Y, const int64_t *ids, const int32_t *assign) {
  if (!ix || n < 0) return ORC_EINVAL;
  if (!ix->has_C) return ORC_ESTATE;
  if (n == 0) return ORC_OK;
  int32_t *a = (int32_t *)malloc((size_t)n * sizeof(int32_t));
  if (assign) memcpy(a, assign, (size_t)n * sizeof(int32_t));
  else orc_assign(ix, n, Y, a);

  /* Would the pool overflow?  Count the new blocks first so a failing batch
   * leaves no trace. */
  {
    int64_t *extra = (int64_t *)calloc((size_t)ix->nlist, sizeof(int64_t));
    for (int64_t i = 0; i < n; ++i) extra[a[i]]++;
    int64_t need = 0;
    for (int k = 0; k < ix->nlist; ++k) {
      int64_t after = (ix->L[k].n + extra[k] + ix->T_m - 1) / ix->T_m;
      need += after - ix->L[k].nchain;
    }
    free(extra);
    if (need > (ix->npool - ix->cur_P) + ix->nfree) { free(a); return ORC_EPOOL; }
  }

  uint8_t *codes = NULL;
  if (ix->pq_m) {
    codes = (uint8_t *)malloc((size_t)n * ix->pq_m);
    orc_pq_encode(ix, n, Y, codes);
  }
  int64_t gid = ix->ntotal;             /* running total: base of the new ids */
  for (int64_t i = 0; i < n; ++i) {
    int k = a[i];
    orc_list *l = &ix->L[k];
    int64_t did = l->n;                 /* atomicAdd(nl_k, 1) */
    int64_t mid = did / ix->T_m, moff = did % ix->T_m;
    if (mid >= l->nchain) {             /* the chain has no block for this slot yet */
      /* only the first slot of a block can open it */
      if (moff != 0) { free(a); free(codes); return ORC_EINVAL; }
      int32_t b;
      if (take_block(ix, &b) != ORC_OK) { free(a); free(codes); return ORC_EPOOL; }
      if (l->nchain == l->chain_cap) {
        l->chain_cap = l->chain_cap ? 2 * l->chain_cap : 4;
        l->chain = (int32_t *)realloc(l->chain, (size_t)l->chain_cap * sizeof(int32_t));
      }
      ix->owner[b] = k; ix->seq[b] = (int32_t)l->nchain;
      l->chain[l->nchain++] = b;        /* link behind the chain's last block */
    }
    list_reserve(l, ix->d, ix->pq_m, did + 1);
    l->ids[did] = ids ? ids[i] : gid + i;
    if (ix->pq_m) memcpy(l->codes + (size_t)did * ix->pq_m, codes + (size_t)i * ix->pq_m, (size_t)ix->pq_m);
    else
      for (int j = 0; j < ix->d; ++j)
        l->x[(size_t)did * ix->d + j] = stored_value(ix->storage, Y[(size_t)i * ix->d + j]);
    l->n = did + 1;
    l->online++;
  }
  ix->ntotal += n;

  /* Rearrangement trigger, list by list (single-threaded part of the
   * Insertion algorithm). */
  if (ix->T_mp > 0)
    for (int k = 0; k < ix->nlist; ++k)
      if (ix->L[k].online > ix->T_mp) orc_rearrange(ix, k);
  free(a);
  free(codes);
  return ORC_OK;
}

/* ------------------------------------------------------------------ search */

typedef struct { double s; int64_t id; } cand;

static int g_metric_for_sort; /* qsort has no context argument; set per call, per thread */
#pragma omp threadprivate(g_metric_for_sort)

static int cand_cmp(const void *pa, const void *pb) {
  const cand *a = (const cand *)pa, *b = (const cand *)pb;
  if (a->s != b->s) return better(g_metric_for_sort, a->s, b->s) ? -1 : 1;
  return (a->id > b->id) - (a->id < b->id);
}

/* The nprobe most relevant lists of one query, best first. */
static void probe_lists(const orc_index *ix, const float *q, int nprobe, int32_t *out) {
  cand *cs = (cand *)malloc((size_t)ix->nlist * sizeof(cand));
  for (int c = 0; c < ix->nlist; ++c) {
    cs[c].s = coarse_score(ix->metric, ix->d, q, ix->C + (size_t)c * ix->d);
    cs[c].id = c;
  }
  g_metric_for_sort = ix->metric;
  qsort(cs, (size_t)ix->nlist, sizeof(cand), cand_cmp);
  for (int p = 0; p < nprobe; ++p) out[p] = (int32_t)cs[p].id;
  free(cs);
}

int orc_probe(const orc_index *ix, int64_t nq, const float *Q, int nprobe, int32_t *out) {
  if (!ix || nprobe < 1 || nprobe > ix->nlist) return ORC_EINVAL;
  if (!ix->has_C) return ORC_ESTATE;
#pragma omp parallel for schedule(dynamic, 4)
  for (int64_t i = 0; i < nq; ++i)
    probe_lists(ix, Q + (size_t)i * ix->d, nprobe, out + (size_t)i * nprobe);
  return ORC_OK;
}

/* Top-k of the probed lists.  out_dist [nq][k] double, out_ids [nq][k].
 * Queries are independent; the loop may run on several cores. */
int orc_search(const orc_index *ix, int64_t nq, const float *Q, int k, int nprobe,
               double *out_dist, int64_t *out_ids) {
  if (!ix || k < 1 || nprobe < 1 || nprobe > ix->nlist || nq < 0) return ORC_EINVAL;
  if (!ix->has_C) return ORC_ESTATE;
#pragma omp parallel for schedule(dynamic, 4)
  for (int64_t i = 0; i < nq; ++i) {
    const float *q = Q + (size_t)i * ix->d;
    int32_t *pl = (int32_t *)malloc((size_t)nprobe * sizeof(int32_t));
    probe_lists(ix, q, nprobe, pl);
    int64_t total = 0;
    for (int p = 0; p < nprobe; ++p) total += ix->L[pl[p]].n;
    cand *cs = (cand *)malloc((size_t)(total > 0 ? total : 1) * sizeof(cand));
    int64_t m = 0;
    double *lut = NULL;  /* [M][256]: query's sub-vector against every codebook entry */
    if (ix->pq_m) {
      const int M = ix->pq_m, ds = ix->d / M;
      lut = (double *)malloc((size_t)M * 256 * sizeof(double));
      for (int s = 0; s < M; ++s)
        for (int c = 0; c < 256; ++c)
          lut[(size_t)s * 256 + c] = fine_score(ix->metric, ds, ix->CB + ((size_t)s * 256 + c) * ds, q + (size_t)s * ds);
    }
    for (int p = 0; p < nprobe; ++p) {
      const orc_list *l = &ix->L[pl[p]];
      for (int64_t e = 0; e < l->n; ++e) {
        if (ix->pq_m) {
          double acc = 0.0;
          for (int s = 0; s < ix->pq_m; ++s) acc = acc + lut[(size_t)s * 256 + l->codes[(size_t)e * ix->pq_m + s]];
          cs[m].s = acc;
        } else {
          cs[m].s = fine_score(ix->metric, ix->d, l->x + (size_t)e * ix->d, q);
        }
        cs[m].id = l->ids[e];
        ++m;
      }
    }
    free(lut);
    g_metric_for_sort = ix->metric;
    qsort(cs, (size_t)m, sizeof(cand), cand_cmp);
    for (int r = 0; r < k; ++r) {
      if (r < m) { out_dist[(size_t)i * k + r] = cs[r].s; out_ids[(size_t)i * k + r] = cs[r].id; }
      else {
        out_dist[(size_t)i * k + r] = ix->metric == ORC_L2 ? INFINITY : -INFINITY;
        out_ids[(size_t)i * k + r] = -1;
      }
    }
    free(cs); free(pl);
  }
  return ORC_OK;
}

/* ----------------------------------------------------------- introspection */

int64_t orc_ntotal(const orc_index *ix) { return ix->ntotal; }
int64_t orc_list_size(const orc_index *ix, int k) { return ix->L[k].n; }
int64_t orc_list_blocks(const orc_index *ix, int k) { return ix->L[k].nchain; }
int64_t orc_list_online(const orc_index *ix, int k) { return ix->L[k].online; }
int64_t orc_blocks_in_use(const orc_index *ix) { return ix->cur_P - ix->nfree; }
int64_t orc_cur_P(const orc_index *ix) { return ix->cur_P; }
int64_t orc_nfree(const orc_index *ix) { return ix->nfree; }
int64_t orc_n_rearrange(const orc_index *ix) { return ix->n_rearrange; }

/* Logical content of list k in list order: ids [n], x [n][d]. */
void orc_list_export(const orc_index *ix, int k, int64_t *ids, float *x) {
  const orc_list *l = &ix->L[k];
  if (ids) memcpy(ids, l->ids, (size_t)l->n * sizeof(int64_t));
  if (x) memcpy(x, l->x, (size_t)l->n * ix->d * sizeof(float));
}

/* Codes of list k in list order: codes [n][M]. */
void orc_list_export_codes(const orc_index *ix, int k, int64_t *ids, uint8_t *codes) {
  const orc_list *l = &ix->L[k];
  if (ids) memcpy(ids, l->ids, (size_t)l->n * sizeof(int64_t));
  if (codes && ix->pq_m) memcpy(codes, l->codes, (size_t)l->n * ix->pq_m);
}

void orc_list_chain(const orc_index *ix, int k, int32_t *chain) {
  memcpy(chain, ix->L[k].chain, (size_t)ix->L[k].nchain * sizeof(int32_t));
}

/* Header jumps of list k: transitions of the chain whose two blocks are not
 * physical neighbours. */
int64_t orc_list_jumps(const orc_index *ix, int k) {
  const orc_list *l = &ix->L[k];
  int64_t j = 0;
  for (int64_t t = 1; t < l->nchain; ++t) j += (l->chain[t] != l->chain[t - 1] + 1);
  return j;
}

/* Where entry did of list k lives: physical block and offset inside it. */
void orc_slot(const orc_index *ix, int k, int64_t did, int32_t *block, int64_t *moff) {
  *block = ix->L[k].chain[did / ix->T_m];
  *moff = did % ix->T_m;
}

/* Bytes of pool memory held by blocks in use, for a block of
 * header_bytes + T_m * (8 + 4 d) bytes. */
int64_t orc_pool_bytes_in_use(const orc_index *ix, int64_t header_bytes) {
  return orc_blocks_in_use(ix) * (header_bytes + ix->T_m * (8 + 4 * (int64_t)ix->d));
}

int orc_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
