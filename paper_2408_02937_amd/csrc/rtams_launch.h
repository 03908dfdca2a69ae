// Host-callable launchers of the kernels, one translation unit per group.
// Internal to the library.
#pragma once
#include "rtams_dev.h"

namespace rtams {

// Work items of the scan of one request.  The items are ordered by list; each
// XCD owns a contiguous range of them.
struct ScanQueues {
  uint32_t begin[9];    // XCD x owns items begin[x] .. begin[x+1]-1
  uint32_t seg_groups;  // 64-vector groups per work item
  // Long scans on the matrix cores: an XCD that has run out of its own items takes items of the others
  // from the back of their ranges (all of these words are zero when the request starts).
  uint32_t back[8];     // items taken from the back of XCD y's range so far
  uint32_t done_mask;   // bit y: nothing is left to take from XCD y
  uint32_t pad[13];
};
static_assert(sizeof(ScanQueues) == 32 * 4, "the request's clearing pass covers the queue words");

// The scan keeps, for every query, only the candidates that are not worse than
// the query's BOUND (the k-th best score of a sample of its candidates, set
// before the scan starts): they are appended to the query's survivor records.

// Per-request scratch of one stream resource (device pointers into its slice).
struct SearchScratch {
  double *scores;       // [max_batch][nlist] coarse scores in the fixed double arithmetic
  float *approx;        // [max_batch][nlist] approximate coarse scores from the matrix cores
  int32_t *probe_list;  // [max_batch][max_nprobe]
  uint32_t *probe_len;  // [max_batch][max_nprobe] list lengths as seen by this request
  unsigned long long *qbase;  // [max_batch] start of the query's slice of rec_key / rec_pos
  uint32_t *qtotal;     // [max_batch] candidates of the query
  uint32_t *bound;      // [max_batch] key of the score the scan compares with
  float *qnorm;         // [max_batch] squared norms of the queries (norm form of the squared distance)
  u32x4 *qsplit;        // [max_batch][dgroups][2] the queries as bf16 halves, for the matrix-core coarse scores
  uint32_t *rec_cnt;    // [max_batch] survivors recorded so far
  unsigned long long *cursor; // bump pointer into the survivor records
  uint32_t *list_cnt;   // [nlist] queries probing each list
  uint32_t *pair_start; // [nlist] where the pairs of a probed list start in `grouped`
  uint32_t *pair_slot;  // [max_batch][max_nprobe] rank of the pair among the pairs of its list
  uint32_t *grouped;    // [max_batch * max_nprobe] pairs (query << 10 | probe) grouped by list
  uint4 *plist;         // [min(nlist, max_batch * max_nprobe)] per probed list, in list order: {list, first pair,
                        // pairs, length as seen by the grouping step}
  uint32_t *pistart;    // [as plist] first work item of the list
  uint4 *tile_desc;     // [item_cap] {list, first pair of the tile, pairs of the tile, segment} per item
  uint32_t item_cap;
  ScanQueues *queues;   // work items of this request, split into one queue per XCD
  float *lut;           // [max_batch][pq_m][256] sub-scores of the queries against the codebooks (PQ lists)
  uint32_t *rec_key;    // survivors: key of the score (smaller is better) ...
  uint32_t *rec_pos;    // ... and its place in the pool (slot_of)
  unsigned long long cand_cap;  // entries of each of the two arrays
  // The reserve shared by all resources, cut into chunks of equal size.  A request whose queries do not
  // all fit into the slice leases ONE chunk (the first query in need takes it, the others share it);
  // queries placed there carry bit 63 in their qbase; the request's last selection workgroup returns it.
  uint32_t *ovf_leased;         // [ovf_chunks] central: 0 free, 1 leased
  uint32_t ovf_chunks;
  unsigned long long ovf_chunk_cap;  // entries of a chunk (in each of the two arrays)
  uint32_t *ovf_key, *ovf_pos;  // central: [ovf_chunks * ovf_chunk_cap] each
  uint32_t *req_chunk;          // this resource's request: 0 none, 1 + the chunk it holds
  uint32_t *req_done;           // selection workgroups of the request that have finished
  unsigned long long *req_cursor;  // entries of the chunk handed out to the request's queries
};

constexpr unsigned long long kInOverflow = 1ull << 63;  // flag in SearchScratch::qbase
constexpr int kMaxOverflowChunks = 32;

constexpr int kScanTileQueries = 8;  // queries that share one pass over a list

// What a 64 x 128 tile of approximate coarse scores is reduced to, per row: the
// tile's smallest score and the columns within the error band of it.
constexpr int kTileCands = 4;
struct TileCands {
  int32_t tiles;   // tiles per row = ceil(nlist / 128)
  float *tmin;     // [rows][tiles]
  uint32_t *cnt;   // [rows][tiles] columns within the band (may exceed kTileCands: then all 128 are rescored)
  int32_t *col;    // [rows][tiles][kTileCands]
  float *val;      // [rows][tiles][kTileCands]
};

// Scratch of the insertion path (lives in the pool's control region).
struct InsertScratch {
  int32_t *assign;   // [max_add_batch] list of each vector
  uint32_t *did;     // [max_add_batch] position inside the list
  double *pscore;    // [part_cap] best score per (vector, centroid split)
  int32_t *pidx;     // [part_cap]
  size_t part_cap;
  TileCands tiles;   // per (row, tile of 128 centroids) digest of the approximate scores of one sub-round
  u32x4 *ysplit;     // [tile_rows][dgroups][2] the vectors of one sub-round as bf16 halves
  float *ynorm;      // [tile_rows] their squared norms
  int64_t tile_rows; // rows one sub-round may hold
};

// Scratch of one rearrangement round (lives in the pool's control region).
struct RearrangeHead {
  int32_t list;    // list being rearranged, -1 none
  uint32_t count;  // moves of this round
  uint32_t nvict;  // occupants that had to be moved out of the way
  uint32_t done;   // the round reaches the end of the chain
  uint32_t state;  // after the round: 0 the list is contiguous (or nothing was to do), 1 another round is owed,
                   // 2 stalled: no spare block in the pool
  uint32_t cursor; // where the search for the next exceeding list starts (kept from round to round)
};
struct RearrangeScratch {
  RearrangeHead *head;
  uint32_t cap;        // moves per round
  uint32_t *mv_t;      // [cap] chain position of each move, ascending
  uint32_t *kind;      // [cap] what sits at the target: 0 never handed out, 1 free, 2 a block in use
  uint32_t *vic_rank;  // [cap] rank among the occupants in use
  uint32_t *vic_new;   // [cap] block the occupant is copied to
  uint32_t *old_src;   // [cap] block the list gives up
  int32_t *vic_list;   // [cap] owner of the occupant
  int32_t *vic_seq;    // [cap] its position in the owner's chain
};

// coarse.hip ---------------------------------------------------------------
int coarse_vt(int d);                      // vectors per workgroup for this dimension
int coarse_splits(const Dev &D, int64_t n, size_t part_cap);
// full score matrix scores[n][nlist]
void launch_coarse_scores(const Dev &D, int64_t n, const float *Y, double *scores,
                          unsigned long long *cursor_to_clear, uint32_t *zero, int zero_n, hipStream_t s);
// per (vector, split) best centroid
void launch_coarse_argmin(const Dev &D, int64_t n, const float *Y, int splits, double *pscore,
                          int32_t *pidx, hipStream_t s);

// coarse_mfma.hip ------------------------------------------------------------
// When the matrix-core filter runs in front of the exact coarse arithmetic: the
// batch has to be a dense contraction large enough to repay the extra kernel and
// the refinement (measured crossovers on MI355X, d = 128 and 768: about 1 M (query,
// centroid) pairs for a search and for an assignment alike).
inline bool mfma_pays_for_search(int64_t nq, int64_t nlist) { return nq >= 32 && nq * nlist >= (int64_t)1 << 20; }
// (an assignment used to pay from half as many pairs where there are 8192 centroids or more; since the
// exact kernel takes two centroids to a thread it does not: 64 vectors against 8,192 x 768 centroids
// are assigned at 0.91 M vectors/s by the exact kernel alone and at 0.78 M through the filter)
inline bool mfma_pays_for_assign(int64_t m, int64_t nlist) { return m >= 32 && m * nlist >= (int64_t)1 << 20; }
// Twice the error bound of an approximate score, for a vector of squared norm |y|^2 (norms = |y|^2 + max |c|^2):
// the exact best lies among the centroids whose approximation is within this of the smallest one.
__host__ __device__ inline float coarse_band(int d, float norms) {
  return (8.f * (float)(d + 4) * 5.9604645e-8f + 8.f * 1.52587890625e-5f) * norms;
}
void launch_centroid_norms(const Dev &D, hipStream_t s);  // and the centroids' split form
void launch_centroid_transpose(const Dev &D, hipStream_t s);  // the copy the exact coarse kernel streams
// (`split` takes the n rows as bf16 halves, [n][dgroups][2] 16-byte words; `norms` their n squared norms)
void launch_coarse_mfma(const Dev &D, int64_t n, const float *Y, u32x4 *split, float *approx,
                        unsigned long long *cursor_to_clear, uint32_t *zero, int zero_n, hipStream_t s);
int coarse_tiles(const Dev &D);
void launch_coarse_tiles(const Dev &D, int64_t n, const float *Y, u32x4 *split, float *norms, const TileCands &tc,
                         hipStream_t s);
void launch_assign_refine(const Dev &D, int64_t n, const float *Y, const TileCands &tc, bool reserve,
                          int32_t *assign, uint32_t *did, hipStream_t s);

// insert.hip -----------------------------------------------------------------
void launch_reserve(const Dev &D, int64_t n, int splits, const InsertScratch &S, bool reserve,
                    int32_t *assign_out, hipStream_t s);
// Positions for a batch whose lists are already in S.assign, in the order of the batch (one thread per list).
void launch_reserve_ordered(const Dev &D, int64_t n, const InsertScratch &S, hipStream_t s);
void launch_open(const Dev &D, hipStream_t s);
void launch_fill(const Dev &D, int64_t n, const float *Y, const int64_t *ids, int64_t id_base,
                 const InsertScratch &S, hipStream_t s);
void launch_publish(const Dev &D, uint32_t call_seq, hipStream_t s);

// probe.hip, group.hip, scan.hip, pq_scan.hip, select.hip ---------------------
void launch_probe_plan(const Dev &D, int64_t nq, int nprobe, int max_nprobe, const SearchScratch &S,
                       const float *Q, bool from_approx, int32_t *probe_out, hipStream_t s);
// One launch does three things side by side: one workgroup cuts the scan into work
// items, one groups the pairs by list, one per query sets the query's bound.
// (Quantised lists are scanned per query: only the bounds are set.)
void launch_group(const Dev &D, int64_t nq, int nprobe, int max_nprobe, int k, const float *Q,
                  int item_budget, const SearchScratch &S, hipStream_t s);
void launch_scan(const Dev &D, int64_t nq, int nprobe, int max_nprobe, const float *Q, int item_budget,
                 const SearchScratch &S, hipStream_t s);
// the scan of flat float lists on the matrix cores (launch_scan hands such requests on to it)
struct ScanShape;
void launch_scan_mm(const Dev &D, const ScanShape &sh, int max_nprobe, const float *Q, const SearchScratch &S,
                    hipStream_t s);
// the scan over product-quantiser codes (launch_scan hands quantised lists on to it)
void launch_pq_scan(const Dev &D, int64_t nq, int nprobe, int max_nprobe, int item_budget,
                    const SearchScratch &S, hipStream_t s);
void launch_select(const Dev &D, int64_t nq, int k, int nprobe, int max_nprobe, const float *Q,
                   const SearchScratch &S, float *out_dist, int64_t *out_ids, hipStream_t s);

// pq.hip -----------------------------------------------------------------------
void launch_pq_fill(const Dev &D, int64_t n, const float *Y, const int64_t *ids, int64_t id_base,
                    const InsertScratch &S, hipStream_t s);
void launch_pq_transpose(const Dev &D, hipStream_t s);  // after the codebooks changed
void launch_pq_export(const Dev &D, int list, int64_t n, int64_t *ids, uint8_t *codes, hipStream_t s);

// rearrange.hip --------------------------------------------------------------
void launch_rearr_plan(const Dev &D, const RearrangeScratch &R, int list, hipStream_t s);
void launch_rearr_step(const Dev &D, const RearrangeScratch &R, int phase, hipStream_t s);
void launch_rearr_release(const Dev &D, const RearrangeScratch &R, hipStream_t s);

// maint.hip ------------------------------------------------------------------
void launch_export(const Dev &D, int list, int64_t n, int64_t *ids, float *vecs, hipStream_t s);
void launch_chain_copy(const Dev &D, int list, int32_t *out, hipStream_t s);
void launch_list_info(const Dev &D, int list, int32_t *out4, hipStream_t s);
void launch_validate(const Dev &D, int32_t *result2, hipStream_t s);
void launch_copy_plain(void *dst, const void *src, size_t bytes, hipStream_t s);
void launch_read_plain(const void *src, size_t bytes, float *sink, hipStream_t s);

}  // namespace rtams
