/*
 * rtams.h - C ABI of the MI355X block-based inverted-list (IVF-Flat) index with
 * real-time insertion, after arXiv 2408.02937 ("A Real-Time Adaptive
 * Multi-Stream GPU System for Online Approximate Nearest Neighborhood Search").
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 * Pointers named d_* are DEVICE pointers (gfx950 HBM); everything else is host
 * memory.  `hip_stream` is a hipStream_t passed as void* (NULL = the default
 * stream).  add / search / rearrange / set_centroids only ENQUEUE work on that
 * stream and return; inputs must stay alive, and outputs are valid, once the
 * caller has synchronised the stream.  The library owns no device memory: the
 * block pool and the search scratch are the caller's (section "Memory Block
 * Based Real-time Vector Insertion Algorithm": one central pool, pre-split
 * into blocks; section "Stream-Cached Multi-Stream Execution", consideration
 * 1: no allocation or release while serving).  After rtams_create no entry
 * point allocates or frees device memory.
 * Every function returns RTAMS_OK or a negative rtams_status; nothing throws
 * or aborts across this boundary.  rtams_last_error() gives a thread-local
 * description of the last failure on the calling thread.
 */
#ifndef RTAMS_H
#define RTAMS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rtams_index rtams_index; /* opaque, host side */

enum rtams_metric {
  RTAMS_L2 = 0, /* squared Euclidean distance, smaller is better */
  RTAMS_IP = 1  /* inner product, larger is better */
};

enum rtams_status {
  RTAMS_OK = 0,
  RTAMS_EINVAL = -1,  /* bad argument */
  RTAMS_ESTATE = -2,  /* not in this state: centroids or codebooks not set yet, or set too late */
  RTAMS_EPOOL = -3,   /* the block pool cannot hold the blocks this call may need */
  RTAMS_EBUSY = -4,   /* every stream resource is in flight: request rejected */
  RTAMS_EHIP = -5,    /* a HIP runtime call failed */
  RTAMS_ESCRATCH = -6, /* a search needed more candidate scratch than its resource and the shared reserve hold */
  RTAMS_ENOSPARE = -7  /* a rearrangement found no spare block in the pool to move a block through: the chains
                          it could not compact are as they were, Exceed() keeps holding for their lists */
};

/* What a flat list keeps of each coordinate (a cheaper step towards the quantised lists: the
 * paper stores 32-bit floats).  A vector joins the list of its nearest centroid as it is given;
 * the list keeps, returns (rtams_list_export) and scans the converted vector.  F16: IEEE half
 * precision, round to nearest even, overflow to infinity; d a multiple of 8.  U8: rounded to the
 * nearest integer (ties to even) and clamped to 0..255, NaN becomes 0 — byte-valued data is kept
 * exactly; d a multiple of 16.  Scores are fp32 arithmetic on the converted values, as for F32. */
enum rtams_storage { RTAMS_F32 = 0, RTAMS_F16 = 1, RTAMS_U8 = 2 };

typedef struct rtams_config {
  int32_t d;          /* vector dimension, multiple of 4 */
  int32_t nlist;      /* number of inverted lists / centroids */
  int32_t metric;     /* rtams_metric */
  int32_t block_vecs; /* T_m: vectors per memory block, multiple of 64 */
  int64_t rearrange_threshold; /* T_m' of Exceed(): vectors appended to a list since its
                                  last rearrangement; <= 0 never triggers */
  void *d_pool;       /* device memory carved into control data, tables and blocks */
  size_t pool_bytes;  /* at most what holds 2^32 / block_vecs blocks (a search names a candidate by its
                         place in the pool, a 32-bit number): rtams_create says EINVAL beyond that */
  void *d_scratch;    /* device memory: one slice per stream resource, all of one size, then the
                         shared reserve (overflow_bytes) if any */
  size_t scratch_bytes;
  int32_t n_resources;   /* search requests that may be in flight at once (paper: 32) */
  int32_t max_batch;     /* largest nq of one rtams_search call */
  int32_t max_k;         /* largest k, at most 1024 */
  int32_t max_nprobe;    /* largest nprobe, at most 1024 and at most nlist */
  int32_t max_add_batch; /* vectors handled per internal insertion round; larger adds are
                            split into rounds on the same stream */
  int32_t pq_m;          /* 0: the lists hold the vectors (IVF-Flat).  M > 0: they hold
                            product-quantiser codes, M bytes per vector (IVF-PQ): M a
                            multiple of 4, at most 64, dividing d */
  int32_t storage;       /* rtams_storage: what flat lists keep of a vector (pq_m must be 0 for the narrow kinds) */
  size_t overflow_bytes; /* the last overflow_bytes of d_scratch are a reserve shared by all
                            stream resources, cut into chunks of equal size (the paper's overflow
                            chunks from a central pool, Deployment Detail).  A request whose
                            queries' candidates do not all fit into its own slice leases one
                            free chunk for the rest and returns it when it is finished; queries
                            that fit neither the slice nor the chunk (or find every chunk
                            leased) come back empty and raise ESCRATCH.  0: no reserve */
  int32_t overflow_chunks; /* how many chunks, 1..32; 0 means 4 */
} rtams_config;

typedef struct rtams_stats {
  int64_t ntotal;           /* vectors visible to searches */
  int64_t blocks_total;     /* |P| */
  int64_t blocks_handed_out;/* cur_P: blocks the bump pointer has passed */
  int64_t blocks_free;      /* blocks on the free list */
  int64_t blocks_in_use;    /* blocks_handed_out - blocks_free */
  int64_t block_bytes;      /* stride of one block: header + ids + vectors */
  int64_t pool_bytes;
  int64_t meta_bytes;       /* control data, centroids and tables in front of the blocks */
  double utilisation;       /* blocks_in_use / blocks_total; the paper alerts above 0.9 */
  int64_t lists_exceeding;  /* lists for which Exceed() currently holds */
  int64_t table_entries_used, table_entries_total;
  int64_t overflow_chunks;         /* chunks of the shared scratch reserve */
  int64_t overflow_chunk_entries;  /* candidate entries one chunk holds */
  int64_t overflow_chunks_leased;  /* chunks held by requests not yet finished */
  int64_t rearrangement_state;     /* of the last rearrangement round: 0 its list is contiguous (or nothing was to
                                      do), 1 another round is owed (a round moves as many blocks as the pool has
                                      spare blocks for, at most 4096), 2 stalled: no spare block at all */
  int64_t add_waits;               /* times rtams_add waited for the data stream to learn how many blocks are left
                                      (what the device reports at every publication did not do) */
} rtams_stats;

/* Bytes of pool needed for `blocks` blocks under this configuration (d_pool and
 * pool_bytes of cfg are ignored).  0 on bad arguments. */
size_t rtams_pool_bytes_for(const rtams_config *cfg, int64_t blocks);

/* Bytes of scratch one stream resource needs so that a search of max_batch
 * queries may score `candidates_per_query` list entries per query (8 bytes
 * per entry: key and position of those that survive the pruning bound, with
 * room for all).  A request whose queries have more candidates than that in
 * total leases a chunk of the shared reserve for the rest (overflow_bytes: 256
 * bytes plus 8 per entry, over overflow_chunks chunks), and fails with ESCRATCH
 * (rtams_poll_error) for the queries that fit neither. */
size_t rtams_scratch_bytes_for(const rtams_config *cfg, int64_t candidates_per_query);

/* Bytes of the shared reserve (the overflow_bytes of the configuration, to be added to d_scratch behind
 * the resources' slices) for `chunks` chunks of `candidates_per_chunk` candidate entries each: the
 * lease words and, per chunk, room for the key and the position of every entry.  0 on bad arguments
 * (chunks outside 1..32, a negative count). */
size_t rtams_overflow_bytes_for(int32_t chunks, int64_t candidates_per_chunk);

/* Creates the index over caller-owned device memory (both regions 256-byte
 * aligned).  Lays out the pool, clears its control data, creates the stream
 * resources.  Synchronous. EINVAL when a size does not fit (rtams_last_error()
 * says which). */
int rtams_create(const rtams_config *cfg, rtams_index **out);

/* Waits for the work this index enqueued, releases host resources.  The
 * caller's device memory is left as it is. */
int rtams_destroy(rtams_index *ix);

/* Copies the centroids ([nlist][d] row-major fp32, device) into the pool.
 * The paper takes them from k-means over the offline set (Insertion
 * algorithm, inputs); producing them is the caller's business.  May be called
 * once, before the first add. */
int rtams_set_centroids(rtams_index *ix, const float *d_centroids, void *hip_stream);

/* Product-quantised lists (pq_m > 0 only; the paper names IVF-PQ beside
 * IVF-Flat as a kind of list its blocks hold, without spelling it out; this is
 * the textbook method).  d_codebooks [pq_m][256][d / pq_m] fp32, copied into
 * the pool; training them is outside this library.  A vector is coded as it is
 * (not its residual to the coarse centroid): code m is the entry of codebook m
 * nearest to its m-th sub-vector in squared Euclidean distance (both metrics),
 * ties to the lowest entry.  A search scores a coded vector by the sum over m
 * of the squared distance (L2) or inner product (IP) between the query's m-th
 * sub-vector and the entry its code names.  ESTATE once vectors are in, or when
 * pq_m is 0; add and search return ESTATE until the codebooks are set. */
int rtams_set_codebooks(rtams_index *ix, const float *d_codebooks, void *hip_stream);

/* Insertion algorithm of the paper: nearest centroid of each vector, atomic
 * reservation of the next slot of that list (did -> block did / T_m, offset
 * did % T_m), lock-free opening and linking of the blocks that do not exist
 * yet, in-place fill in the interleaved layout, and the Exceed() test.
 * d_vecs [n][d] row-major fp32; d_ids [n] int64 or NULL (then the ids are
 * ntotal .. ntotal+n-1 at the time of the call).  The batch becomes visible to
 * searches as a whole, after its last vector is written.  All adds (and
 * rearrangements) are ordered one after another: the paper's single data
 * stream; a call on another stream than the previous one is ordered behind it
 * with an event.  EPOOL (nothing enqueued) when the pool might overflow:
 * the call counts the blocks the batch may open at most (one per touched list
 * plus the full ones) against the blocks left, which it takes from what the
 * device reports to pinned host memory whenever a batch is published, less
 * what the batches enqueued since may open.  Only when that estimate falls
 * short does the call WAIT for the data stream and read the allocator's own
 * counters (rtams_stats.add_waits counts these waits) before it says EPOOL. */
int rtams_add(rtams_index *ix, int64_t n, const float *d_vecs, const int64_t *d_ids,
              void *hip_stream);

/* Batched search (paper, introduction: the lists of the nprobe clusters most
 * relevant to the query are scanned, the top-k returned; exact distances).
 * d_queries [nq][d]; d_out_dist [nq][k] fp32 (squared L2, or inner product);
 * d_out_ids [nq][k] int64.  Rows are ordered best first, ties by ascending id;
 * missing results are id -1 with +inf (L2) / -inf (IP).  Takes one stream
 * resource (scratch slice) for the duration of the request, Multi Stream
 * Execution algorithm; EBUSY (nothing enqueued) when none is free.  Any number
 * of host threads may search concurrently, each on its own stream.  A search
 * sees whole insertion batches only. */
int rtams_search(rtams_index *ix, int64_t nq, const float *d_queries, int32_t k, int32_t nprobe,
                 float *d_out_dist, int64_t *d_out_ids, void *hip_stream);

/* rtams_search for callers that cannot allocate and have no scratch of their own to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same answers,
 * same kernels; the request's scratch is not a slice of the caller's d_scratch but an array in the device
 * image of this library (32 MiB on every GPU the library runs on, held until the process ends; its
 * address on the index's device is looked up once, in rtams_create).  Neither this call nor anything it
 * launches allocates or frees memory.  Limits: nq at most 64 (EINVAL beyond; also EINVAL when the fixed
 * part of a request of this index, which grows with nlist and max_nprobe, does not fit the array); a
 * query's candidates beyond what the array holds behind that fixed part (about two million entries at
 * nlist 16384, more with fewer lists) make that query come back empty with ESCRATCH, as for rtams_search
 * without a reserve.  Every call on a GPU shares that GPU's array, which keeps the last call's contents
 * (each request clears what it needs cleared): one request at a time.  A second call on the same index
 * before the first has finished is refused with EBUSY; calls through DIFFERENT indexes on one GPU that
 * overlap are not detected and race. */
int rtams_search_noalloc(rtams_index *ix, int64_t nq, const float *d_queries, int32_t k, int32_t nprobe,
                         float *d_out_dist, int64_t *d_out_ids, void *hip_stream);

/* Rearrangement algorithm of the paper: makes the blocks of `list` physically
 * contiguous behind its first block by exchanging blocks with their physical
 * neighbours.  list == -1 handles every list for which Exceed() holds.  The work
 * goes in rounds (a round moves one list's blocks: at most 4096, and no more
 * than the pool has spare blocks to move the displaced occupants through, one
 * at least while a single block is free), and this call WAITS for each round
 * on the stream, because only the device knows whether another is owed; it
 * returns when the chain is contiguous (list >= 0) or no list exceeds (-1).
 * ENOSPARE when the pool has no spare block at all: nothing is lost, the
 * chains concerned are as they were and Exceed() keeps holding for them.
 * rtams_add enqueues ONE round by itself, without waiting, when it finds that
 * Exceed() held after an EARLIER batch was published (the device reports that
 * through a word of pinned host memory).  After the last batch of a burst
 * nothing follows that could carry the round: a caller who wants every
 * exceeding list compacted then calls rtams_rearrange(ix, -1, ...) itself
 * (rtams_pool_stats().lists_exceeding tells whether any is left).
 * Ordered with add on the data stream; searches keep running and see either
 * placement, never a mixture. */
int rtams_rearrange(rtams_index *ix, int32_t list, void *hip_stream);

/* ---- introspection and test hooks; these synchronise the data stream ---- */

int rtams_ntotal(rtams_index *ix, int64_t *out);
int rtams_list_size(rtams_index *ix, int32_t list, int64_t *out);
/* blocks of the list, physical runs ("header jumps" + 1, 0 for an empty list) and
 * vectors appended since its last rearrangement */
int rtams_list_info(rtams_index *ix, int32_t list, int64_t *blocks, int64_t *runs,
                    int64_t *online);
/* Logical content of one list in list order: d_ids [cap] and d_vecs [cap][d]
 * row-major fp32 (either may be NULL; with F16 or U8 storage the vectors as the
 * list keeps them, widened); *n_out = list length; EINVAL if cap is too small. */
int rtams_list_export(rtams_index *ix, int32_t list, int64_t cap, int64_t *d_ids, float *d_vecs,
                      int64_t *n_out, void *hip_stream);
/* Physical block numbers of the list's chain, in logical order (host array). */
int rtams_list_chain(rtams_index *ix, int32_t list, int64_t cap, int32_t *chain, int64_t *n_out);
/* Visible length of every list at once (host array [nlist]). */
int rtams_list_sizes(rtams_index *ix, int64_t *out);
int rtams_pool_stats(rtams_index *ix, rtams_stats *out);
/* Device-side check of the block structure (chain lengths, header links, table
 * against headers, no block owned twice, free list disjoint from chains).
 * Returns RTAMS_OK or RTAMS_EINVAL with the violation in rtams_last_error(). */
int rtams_validate(rtams_index *ix, void *hip_stream);
/* Probed lists of each query, best first (d_out [nq][nprobe] int32, device). */
int rtams_probe(rtams_index *ix, int64_t nq, const float *d_queries, int32_t nprobe,
                int32_t *d_out, void *hip_stream);
/* Nearest centroid of each vector (d_out [n] int32, device), nothing inserted. */
int rtams_assign(rtams_index *ix, int64_t n, const float *d_vecs, int32_t *d_out,
                 void *hip_stream);

/* Sticky asynchronous error raised by a kernel; RTAMS_OK if none.  Does not
 * synchronise.  EPOOL (a batch found the pool exhausted on the device: the batch
 * was dropped as a whole and the index takes no further vectors) comes first
 * and stays.  ESCRATCH (some query of some search had more candidates than its
 * slice and the reserve could take: that query came back empty) concerns
 * searches only, inserts and later searches go on as usual; it stays until
 * rtams_clear_error. */
int rtams_poll_error(rtams_index *ix);
/* Forgets an ESCRATCH (not an EPOOL).  Synchronous; call it when no search is
 * in flight, or a failure being raised at that moment may be lost. */
int rtams_clear_error(rtams_index *ix);
const char *rtams_last_error(void);
/* Codes of a product-quantised list in list order: d_ids [cap] int64 (or NULL),
 * d_codes [cap][pq_m] bytes (or NULL), *n_out = entries of the list (at most
 * cap are written).  Synchronises the stream.  ESTATE for flat lists. */
int rtams_list_export_codes(rtams_index *ix, int32_t list, int64_t cap, int64_t *d_ids, uint8_t *d_codes,
                            int64_t *n_out, void *hip_stream);

/* Launch-shape knobs (Stream-Cached Multi-Stream Execution, consideration 2: what a kernel may take
 * of the chip is capped so that several kernels run side by side).  None of them changes a result.
 * EINVAL for an unknown key; values out of a key's range are clamped.  May be called while requests
 * are in flight: a request takes the values it finds when it is enqueued.
 *   "scan_max_items"       most work items one list-scan launch is cut into (a (query, list) pair is
 *                          always at least one); default 32768, at least 1024.
 *   "scan_items_per_pair"  work items per (query, list) pair a small request may be cut into;
 *                          default 8.
 *   "scan_mfma"            flat float lists: whether the scan's dot products run on the matrix cores,
 *                          one workgroup per work item with a tile of up to 32 queries in LDS.  0
 *                          never, 2 always, 1 (default) for requests of 64 queries or more whose tiles
 *                          hold several queries: at least as many (query, list) pairs as lists, or a
 *                          list 16 times as long as the average.
 *   "scan_min_choice"      shortest segment of a list the plan may make a work item of, as the power
 *                          e of 2 << e groups of 64 vectors (0..7); -1 (default) leaves it to the
 *                          scan kernel (2 groups on the vector unit, 8 on the matrix cores).
 *   "scan_byte_weight"     what reading a group of 64 vectors costs, in queries' worth of arithmetic,
 *                          when the work is split over the chip's 8 dies; 0 (default) takes 12 for
 *                          L2 and 24 for inner products.
 *   "scan_exclusive_pairs" / "scan_exclusive_bytes"
 *                          a request's scan queues up behind the previous such scan, whatever streams
 *                          they are on, when the request has at least so many (query, list) pairs
 *                          (default 4096; 0: never) AND those pairs are expected to meet at least so
 *                          many list bytes, lists taken at their average length (default 16 GiB):
 *                          scans of a millisecond or more gain nothing from running side by side.
 *   "scan_steal"           1 (default): in such a long scan on the matrix cores, a die that has run out
 *                          of its share of the work items takes items from the back of another die's
 *                          share; 0: every die scans its own share only.  The result is the same.
 *   "use_mfma"             whether approximate coarse scores from the matrix cores filter the
 *                          centroids before the exact arithmetic decides: 0 never, 1 for batches large
 *                          enough to repay it (default), 2 for every batch of 32 rows or more.
 *   "ordered_add"          0 (default) reserves the positions of a batch inside a list with one atomic
 *                          per vector, in arrival order, as the Insertion algorithm does; 1 hands them
 *                          out in the order of the batch, so that every list holds the sequence that
 *                          inserting the vectors one at a time would give (one thread per list walks
 *                          the batch: slower, meant for checking).  This one changes the ORDER inside
 *                          a list, which the paper leaves to the atomics.
 *   "profile_scan"         see rtams_scan_time (rtams_measure.h). */
int rtams_set_param(rtams_index *ix, const char *key, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* RTAMS_H */
