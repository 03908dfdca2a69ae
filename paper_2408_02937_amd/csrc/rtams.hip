// Host side of the C ABI declared in include/rtams.h: pool layout, stream
// resources, and the enqueue-only entry points.
#include "../../include/rtams.h"
#include "../../include/rtams_measure.h"

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <shared_mutex>

#include "search_common.h"

using namespace rtams;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                  \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess)                                                              \
      return fail(RTAMS_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));          \
  } while (0)

inline size_t up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Byte offsets of everything in front of the blocks.
struct Layout {
  size_t ctrl, hook, centroids, centroids_t, cnorm, csplit, codebooks, codebooks_t, tc_min, tc_cnt, tc_col, tc_val, ins_ysplit, ins_ynorm, tile_rows, reserved_len, visible_len, online, nblk, exceed, seg_dir;
  size_t ins_assign, ins_did, ins_pscore, ins_pidx, part_cap;
  size_t rearr_head, rearr_arrays;
  size_t fixed_end;          // end of the part that does not depend on the block count
  size_t slab, free_stack, mark, blocks;
  size_t block_stride;
  uint32_t ids_off, vec_off;
  uint64_t slab_cap;
  int64_t nblocks;
  size_t total;
};

constexpr size_t kAlign = 256;
constexpr uint32_t kRearrangeCap = 4096;  // block moves per rearrangement round
constexpr size_t kHookBytes = 256;

bool config_ok(const rtams_config *c, bool need_memory) {
  if (!c) return fail(RTAMS_EINVAL, "config is NULL"), false;
  if (c->d <= 0 || c->d % 4 != 0 || c->d > 2048)
    return fail(RTAMS_EINVAL, "d must be a multiple of 4 in 4..2048, got %d", c->d), false;
  if (c->nlist <= 0) return fail(RTAMS_EINVAL, "nlist must be positive"), false;
  if (c->pq_m < 0 || (c->pq_m > 0 && (c->pq_m % 4 != 0 || c->pq_m > 64 || c->d % c->pq_m != 0)))
    return fail(RTAMS_EINVAL, "pq_m must be 0, or a multiple of 4 up to 64 that divides d; got %d", c->pq_m), false;
  if (c->metric != RTAMS_L2 && c->metric != RTAMS_IP) return fail(RTAMS_EINVAL, "unknown metric"), false;
  if (c->storage < RTAMS_F32 || c->storage > RTAMS_U8 || (c->storage != RTAMS_F32 && c->pq_m > 0) ||
      (c->storage == RTAMS_F16 && c->d % 8 != 0) || (c->storage == RTAMS_U8 && c->d % 16 != 0))
    return fail(RTAMS_EINVAL, "storage must be F32, or F16 with d a multiple of 8, or U8 with d a multiple of 16, "
                              "the narrow kinds with pq_m 0; got storage %d, d %d, pq_m %d", c->storage, c->d, c->pq_m), false;
  if (c->block_vecs <= 0 || c->block_vecs % kWave != 0)
    return fail(RTAMS_EINVAL, "block_vecs must be a positive multiple of 64, got %d", c->block_vecs), false;
  if (c->n_resources < 1 || c->n_resources > 256)
    return fail(RTAMS_EINVAL, "n_resources must be in 1..256"), false;
  if (c->max_batch < 1 || c->max_batch > (1 << 20))
    return fail(RTAMS_EINVAL, "max_batch must be in 1..1048576"), false;
  if (c->max_k < 1 || c->max_k > kMaxK) return fail(RTAMS_EINVAL, "max_k must be in 1..%d", kMaxK), false;
  if (c->max_nprobe < 1 || c->max_nprobe > kMaxNprobe || c->max_nprobe > c->nlist)
    return fail(RTAMS_EINVAL, "max_nprobe must be in 1..min(nlist, %d)", kMaxNprobe), false;
  if (c->max_add_batch < 1) return fail(RTAMS_EINVAL, "max_add_batch must be positive"), false;
  if (need_memory) {
    if (!c->d_pool || !c->d_scratch) return fail(RTAMS_EINVAL, "pool and scratch must be given"), false;
    if (((uintptr_t)c->d_pool | (uintptr_t)c->d_scratch) % kAlign)
      return fail(RTAMS_EINVAL, "pool and scratch must be %zu-byte aligned", kAlign), false;
  }
  return true;
}

// Fixed part first; then, given a byte budget (blocks < 0) or a block count, the rest.
void lay_out(const rtams_config *c, int64_t blocks, size_t pool_bytes, Layout *L) {
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = up(o + bytes, kAlign); return at; };
  const size_t nl = (size_t)c->nlist;
  L->ctrl = take(sizeof(Ctrl));
  L->hook = take(kHookBytes);
  L->centroids = take(nl * c->d * sizeof(float));
  L->centroids_t = take(nl * c->d * sizeof(float));
  L->cnorm = take(nl * sizeof(float));
  L->csplit = take(nl * (size_t)((c->d + 31) / 32) * 4 * 32);
  L->codebooks = take(c->pq_m > 0 ? (size_t)256 * c->d * sizeof(float) : 0);
  L->codebooks_t = take(c->pq_m > 0 ? (size_t)256 * c->d * sizeof(float) : 0);
  L->reserved_len = take(nl * 4);
  L->visible_len = take(nl * 4);
  L->online = take(nl * 4);
  L->nblk = take(nl * 4);
  L->exceed = take(nl);
  L->seg_dir = take(nl * kTableSegs * 4);
  L->part_cap = (size_t)c->max_add_batch * 2 > 65536 ? (size_t)c->max_add_batch * 2 : 65536;
  L->ins_assign = take((size_t)c->max_add_batch * 4);
  L->ins_did = take((size_t)c->max_add_batch * 4);
  L->ins_pscore = take(L->part_cap * 8);
  L->ins_pidx = take(L->part_cap * 4);
  {  // tile digests of one insertion sub-round (40 bytes per row and tile): at most 64 MiB, at least 64 rows
    const size_t tiles = (nl + 127) / 128;
    size_t rows = ((size_t)64 << 20) / (tiles * 40);
    const size_t split_row = (size_t)((c->d + 31) / 32) * 4 * 32;  // a vector as bf16 halves: at most 64 MiB of those, too
    if (rows > ((size_t)64 << 20) / split_row) rows = ((size_t)64 << 20) / split_row;
    if (rows > (size_t)c->max_add_batch) rows = (size_t)c->max_add_batch;
    if (rows < 64) rows = 64;
    L->tile_rows = rows;
    L->ins_ysplit = take(rows * split_row);
    L->ins_ynorm = take(rows * 4);
    L->tc_min = take(rows * tiles * 4);
    L->tc_cnt = take(rows * tiles * 4);
    L->tc_col = take(rows * tiles * kTileCands * 4);
    L->tc_val = take(rows * tiles * kTileCands * 4);
  }
  L->rearr_head = take(sizeof(RearrangeHead));
  L->rearr_arrays = take((size_t)kRearrangeCap * 4 * 7);
  L->fixed_end = o;
  L->ids_off = kHeaderBytes;
  L->vec_off = kHeaderBytes + (uint32_t)c->block_vecs * 8u;
  // a vector takes d floats, or pq_m code bytes
  L->block_stride = up((size_t)L->vec_off + (size_t)c->block_vecs * (c->pq_m > 0 ? (size_t)c->pq_m : (size_t)c->d * (c->storage == RTAMS_F16 ? 2 : c->storage == RTAMS_U8 ? 1 : 4)), kAlign);
  if (blocks < 0) {
    // per block: the block itself, 2 table entries, a free-stack entry and a mark
    size_t slack = 4 * kAlign + nl * kTableBase * 4;
    size_t per = L->block_stride + 16;
    blocks = pool_bytes > o + slack ? (int64_t)((pool_bytes - o - slack) / per) : 0;
    if (blocks > 0x7fffffff) blocks = 0x7fffffff;
  }
  L->nblocks = blocks;
  L->slab_cap = 2ull * (uint64_t)blocks + (uint64_t)nl * kTableBase;
  L->slab = take((size_t)L->slab_cap * 4);
  L->free_stack = take((size_t)blocks * 4);
  L->mark = take((size_t)blocks * 4);
  L->blocks = o;
  L->total = o + (size_t)blocks * L->block_stride;
}

struct ScratchLayout {
  size_t scores, approx, probe_list, probe_len, qbase, qtotal, bound, qnorm, qsplit, rec_cnt, cursor, req_words, lut, records, fixed;
  size_t list_cnt, pair_start, pair_slot, grouped, plist, pistart, tile_desc, queues, item_cap;
};

void lay_out_scratch(const rtams_config *c, ScratchLayout *S) {
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = up(o + bytes, kAlign); return at; };
  size_t mb = (size_t)c->max_batch, mp = (size_t)c->max_nprobe;
  S->scores = take(mb * c->nlist * 8);
  S->approx = take(mb * c->nlist * 4);
  S->lut = take(c->pq_m > 0 ? mb * c->pq_m * 256 * 4 : 0);
  S->probe_list = take(mb * mp * 4);
  S->probe_len = take(mb * mp * 4);
  S->qbase = take(mb * 8);
  S->qtotal = take(mb * 4);
  S->bound = take(mb * 4);
  S->qnorm = take(mb * 4);
  S->qsplit = take(mb * (size_t)((c->d + 31) / 32) * 4 * 32);
  S->rec_cnt = take(mb * 4);
  S->cursor = take(8);
  S->req_words = take(16);  // the request's chunk of the shared reserve: chunk, finished workgroups, cursor
  // list_cnt and the queue heads are cleared together at the start of every request
  S->list_cnt = take((size_t)c->nlist * 4);
  S->queues = take(sizeof(ScanQueues));
  const size_t probed = mb * mp < (size_t)c->nlist ? mb * mp : (size_t)c->nlist;  // lists one request can probe
  S->pair_start = take((size_t)c->nlist * 4);
  S->pair_slot = take(mb * mp * 4);
  S->grouped = take(mb * mp * 4);
  S->plist = take(probed * 16);
  S->pistart = take(probed * 4);
  S->item_cap = mb * mp * 4 > 65536 ? mb * mp * 4 : 65536;
  S->tile_desc = take(S->item_cap * 16);
  S->records = o;
  S->fixed = o;
}

// Search scratch for callers that cannot hand any over and must not allocate (rtams_search_noalloc):
// one array in the device image of this library.  Every GPU the library runs on holds its own copy at
// its own address until the process ends; the name below is only a host-side stand-in for the symbol,
// never a device address: host code uses the pointer hipGetSymbolAddress returns for the current device.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kStaticMaxBatch = 64;  // queries of one rtams_search_noalloc call at most
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_static_mutex;
void *g_static_ptr[kMaxDevices] = {};  // per device: where its copy of `scratch` lies

// Address of the current device's copy of the array, resolved once per device with that device current.
int static_scratch_of_current_device(void **out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(RTAMS_EINVAL, "device %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> g(g_static_mutex);
  if (!g_static_ptr[dev]) {
    void *p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(RTAMS_EHIP, "hipGetSymbolAddress returned no address");
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return RTAMS_OK;
}

enum { RES_FREE = 0, RES_BUSY = 1, RES_PENDING = 2 };

struct Resource {
  std::atomic<int> state{RES_FREE};
  hipEvent_t done = nullptr;
  hipEvent_t t0 = nullptr, t1 = nullptr;  // around the grouped scan when profiling is on
  hipEvent_t scan_done = nullptr;         // behind the scan of the slot's request (large requests queue up their scans)
  bool timed = false;
  SearchScratch s{};
};

}  // namespace

struct rtams_index {
  rtams_config cfg{};
  Layout lay{};
  Dev dev{};
  InsertScratch ins{};
  RearrangeScratch rearr{};
  HostMirror *mirror = nullptr;
  char *hook = nullptr;  // device scratch of the introspection calls
  Resource *res = nullptr;  // n_res pooled ones over the caller's scratch, then one over the library's static array
  int n_res = 0;
  bool static_ok = false;    // the static array holds a request of this index
  int static_max_batch = 0;
  bool has_centroids = false;
  std::mutex data_mutex;  // add / rearrange / hooks: the single data stream of the paper
  hipStream_t data_stream = nullptr;
  bool have_data_stream = false;
  hipEvent_t data_done = nullptr;
  // Searches hold this shared while they enqueue; a rearrangement takes it
  // exclusively for the instant in which it fences the searches in flight.
  std::shared_mutex fence_mutex;
  hipEvent_t fence_ev[2] = {nullptr, nullptr};  // table switches of the running rearrangement
  hipEvent_t fence_cur = nullptr;               // what a new search must wait for, or nullptr
  std::atomic<int64_t> ntotal_host{0};   // vectors handed to add so far (written under data_mutex; searches read it for estimates)
  int64_t avail_lb = 0;      // lower bound of the blocks still available in the pool
  // Insertion calls enqueued whose publication the host has not seen yet, with the blocks each may open at most
  // (under data_mutex).  The device reports (number of the last call published, blocks in use) in one word.
  struct PendingAdd { uint32_t seq; int64_t need; };
  std::deque<PendingAdd> pending_adds;
  int64_t pending_need = 0;
  uint32_t add_seq = 0;
  int64_t add_waits = 0;     // times an add had to wait for the data stream to learn how many blocks are left
  std::atomic<int64_t> scan_items_per_pair{8};   // work items the plan may cut per (query, list) pair
  std::atomic<int64_t> scan_max_items{32768};    // ... and per request
  std::atomic<int64_t> profile_scan{0};
  std::atomic<int64_t> timed_scans[3] = {{0}, {0}, {0}};  // timed launches of k_scan, k_scan_mm, k_pq_scan
  bool has_codebooks = false;
  uint32_t *ovf_leased = nullptr;  // device: which chunks of the shared scratch reserve are leased
  uint32_t ovf_chunks = 0;
  unsigned long long ovf_chunk_cap = 0;
  std::atomic<int64_t> ordered_add{0};  // positions inside a list in the order of the batch instead of arrival order
  std::atomic<int64_t> use_mfma{1};  // matrix-core filter in front of the exact coarse arithmetic
  std::atomic<int64_t> scan_mfma{1}; // flat float lists: the scan's dot products on the matrix cores
  std::atomic<int64_t> scan_byte_weight{0};
  std::atomic<int64_t> scan_min_choice{-1};
  // Scans of LONG requests run one after the other, whatever streams they are on: such a scan fills the
  // chip by itself for milliseconds, and two of them side by side only slow each other down (both finish
  // when the sum of their work is done, instead of one after half of it); everything else of a request
  // still overlaps with other requests' scans.  (Consideration 2 of the multi-stream section: what a
  // kernel may take of the chip is limited so that kernels of other streams are not held up.)  Handing
  // the chip from one stream to the next costs some tens of microseconds, which a scan of a
  // millisecond or more does not feel (measured: 2 % of the throughput at 2.7 ms a scan) and shorter
  // ones do (12 % at 0.6 ms, 23 % at 0.12 ms): those overlap freely and fill each other's tails.  A
  // request is long when the list bytes its (query, list) pairs are expected to meet (lists of
  // average length) reach scan_exclusive_bytes.
  std::mutex scan_mutex;
  hipEvent_t scan_tail = nullptr;                 // behind the last large scan enqueued, or nullptr
  std::atomic<int64_t> scan_exclusive_pairs{4096};  // (query, list) pairs from which a request's scan may queue up; 0 never
  std::atomic<int64_t> scan_exclusive_bytes{(int64_t)16 << 30};  // ... and expected list bytes of those pairs from which it does
  std::atomic<int64_t> scan_steal{1};  // such a long scan, on the matrix cores: XCDs that are done take items of the others
  std::mutex prof_mutex;
  double scan_ms = 0.0;      // sum of measured scan-kernel durations
  int64_t scan_launches = 0;
};

namespace {

// 32-bit words cleared at the start of a request: per-list pair counters and, right
// behind them in the slice, the scan queues
int plan_words(const rtams_index *ix) {
  return (int)(((const char *)ix->res[0].s.queues - (const char *)ix->res[0].s.list_cnt) / 4 +
               sizeof(ScanQueues) / 4);
}

// Coarse scores of the queries, probe selection and the plan of the scan.
void coarse_and_plan(rtams_index *ix, int64_t nq, const float *Q, int nprobe, const SearchScratch &S,
                     int32_t *probe_out, hipStream_t s) {
  const Dev &D = ix->dev;
  const int64_t mode = ix->use_mfma.load(std::memory_order_relaxed);  // 0 never, 1 when it pays, 2 from 32 rows
  const bool mfma = mode == 2 ? nq >= 32 : mode == 1 && mfma_pays_for_search(nq, D.nlist);
  if (mfma) launch_coarse_mfma(D, nq, Q, S.qsplit, S.approx, S.cursor, S.list_cnt, plan_words(ix), s);
  else launch_coarse_scores(D, nq, Q, S.scores, S.cursor, S.list_cnt, plan_words(ix), s);
  launch_probe_plan(D, nq, nprobe, ix->cfg.max_nprobe, S, Q, mfma, probe_out, s);
}

int sync_data(rtams_index *ix) {
  if (ix->have_data_stream) HIP_TRY(hipStreamSynchronize(ix->data_stream));
  return RTAMS_OK;
}

// Blocks still available, from what the device last reported: the blocks in use after the insertion
// call it names, less what the calls enqueued after that one may open.  Blocks in use never shrink
// between two publications (a rearrangement round returns the spare blocks it took before the next
// batch runs), so this is a lower bound whichever publication the word is from.  No waiting.
void tighten_pool_bound(rtams_index *ix) {
  const unsigned long long w = ix->mirror->pool_word;  // one aligned 64-bit load
  const uint32_t seen = (uint32_t)(w >> 32), in_use = (uint32_t)w;
  while (!ix->pending_adds.empty() && (int32_t)(seen - ix->pending_adds.front().seq) >= 0) {
    ix->pending_need -= ix->pending_adds.front().need;
    ix->pending_adds.pop_front();
  }
  const int64_t left = (int64_t)ix->dev.nblocks - (int64_t)in_use - ix->pending_need;
  if (left > ix->avail_lb) ix->avail_lb = left;
}

// Orders this call behind the previous work of the data stream.
int enter_data_stream(rtams_index *ix, hipStream_t s) {
  if (ix->have_data_stream && ix->data_stream != s) HIP_TRY(hipStreamWaitEvent(s, ix->data_done, 0));
  ix->data_stream = s;
  ix->have_data_stream = true;
  return RTAMS_OK;
}

// Whatever way a call on the data stream ends, the next one has to find where it ended.
struct DataStreamScope {
  rtams_index *ix;
  hipStream_t s;
  ~DataStreamScope() { (void)hipEventRecord(ix->data_done, s); }
};

// The owner of a resource (state BUSY) collects the scan timing of its last request.
void harvest(rtams_index *ix, Resource &R) {
  if (!R.timed) return;
  R.timed = false;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, R.t0, R.t1) == hipSuccess) {
    std::lock_guard<std::mutex> g(ix->prof_mutex);
    ix->scan_ms += ms;
    ix->scan_launches += 1;
  } else {
    (void)hipGetLastError();
  }
}

// Lock-free hand-out of stream resources: a slot is FREE, BUSY (being filled by
// a host thread) or PENDING (its request is on the GPU; the next taker checks
// the completion event).
int acquire(rtams_index *ix) {
  for (int r = 0; r < ix->n_res; ++r) {
    int st = ix->res[r].state.load(std::memory_order_acquire);
    if (st == RES_FREE) {
      if (ix->res[r].state.compare_exchange_strong(st, RES_BUSY, std::memory_order_acq_rel)) return r;
    } else if (st == RES_PENDING) {
      if (hipEventQuery(ix->res[r].done) == hipSuccess &&
          ix->res[r].state.compare_exchange_strong(st, RES_BUSY, std::memory_order_acq_rel)) {
        harvest(ix, ix->res[r]);
        return r;
      }
    }
  }
  (void)hipGetLastError();  // hipEventQuery leaves hipErrorNotReady behind
  return -1;
}

// Nearest centroid of m vectors (m <= max_add_batch) and, if asked, the slot
// reservation.  A batch that is a large dense contraction gets approximate
// scores on the matrix cores, then exact refinement of what they cannot tell
// apart; smaller batches go through the exact kernel alone.
void assign_round(rtams_index *ix, int64_t m, const float *Y, bool reserve, int32_t *assign_out, hipStream_t s) {
  const Dev &D = ix->dev;
  const int64_t mode = ix->use_mfma.load(std::memory_order_relaxed);  // 0 never, 1 when it pays, 2 from 32 rows
  if (mode == 2 ? m >= 32 : mode == 1 && mfma_pays_for_assign(m, D.nlist)) {
    for (int64_t o = 0; o < m; o += ix->ins.tile_rows) {
      const int64_t mm = m - o < ix->ins.tile_rows ? m - o : ix->ins.tile_rows;
      launch_coarse_tiles(D, mm, Y + (size_t)o * D.d, ix->ins.ysplit, ix->ins.ynorm, ix->ins.tiles, s);
      launch_assign_refine(D, mm, Y + (size_t)o * D.d, ix->ins.tiles, reserve, assign_out + o, ix->ins.did + o, s);
    }
  } else {
    int splits = coarse_splits(D, m, ix->ins.part_cap);
    launch_coarse_argmin(D, m, Y, splits, ix->ins.pscore, ix->ins.pidx, s);
    launch_reserve(D, m, splits, ix->ins, reserve, assign_out, s);
  }
}

int read_ctrl(rtams_index *ix, Ctrl *out) {
  HIP_TRY(hipMemcpy(out, ix->dev.ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost));
  return RTAMS_OK;
}

}  // namespace

static int rearrange_round(rtams_index *ix, int32_t list, hipStream_t s);

extern "C" {

const char *rtams_last_error(void) { return g_err; }

size_t rtams_pool_bytes_for(const rtams_config *cfg, int64_t blocks) {
  if (!config_ok(cfg, false) || blocks < 0) return 0;
  Layout L;
  lay_out(cfg, blocks, 0, &L);
  return up(L.total + 4 * kAlign + (size_t)cfg->nlist * kTableBase * 4, kAlign);
}

size_t rtams_scratch_bytes_for(const rtams_config *cfg, int64_t candidates_per_query) {
  if (!config_ok(cfg, false) || candidates_per_query < 0) return 0;
  ScratchLayout S;
  lay_out_scratch(cfg, &S);
  // key and position of a surviving candidate: 8 bytes each, room for all of them
  return up(S.fixed + 2 * up((size_t)cfg->max_batch * (size_t)candidates_per_query * 4, kAlign), kAlign);
}

size_t rtams_overflow_bytes_for(int32_t chunks, int64_t candidates_per_chunk) {
  if (chunks < 1 || chunks > kMaxOverflowChunks || candidates_per_chunk < 0) return 0;
  // the lease words, then two arrays (keys, positions) cut into chunks of whole 256-byte units
  return kAlign + 2 * (size_t)chunks * up((size_t)candidates_per_chunk * 4, kAlign);
}

int rtams_create(const rtams_config *cfg, rtams_index **out) {
  if (!out) return fail(RTAMS_EINVAL, "out is NULL");
  *out = nullptr;
  if (!config_ok(cfg, true)) return RTAMS_EINVAL;
  Layout L;
  lay_out(cfg, -1, cfg->pool_bytes, &L);
  if (L.nblocks < 1 || L.total > cfg->pool_bytes)
    return fail(RTAMS_EINVAL, "pool of %zu bytes holds no block (control data needs %zu, a block %zu)",
                cfg->pool_bytes, L.fixed_end, L.block_stride);
  // a search names a surviving candidate by its place in the pool, a 32-bit number
  if ((uint64_t)L.nblocks * (uint64_t)cfg->block_vecs > (1ull << 32))
    return fail(RTAMS_EINVAL, "pool of %zu bytes holds %lld blocks of %d vectors: more than 2^32 places; pass at most %zu bytes",
                cfg->pool_bytes, (long long)L.nblocks, cfg->block_vecs,
                rtams_pool_bytes_for(cfg, (int64_t)((1ull << 32) / (uint64_t)cfg->block_vecs)));
  ScratchLayout SL;
  lay_out_scratch(cfg, &SL);
  if (cfg->overflow_bytes > cfg->scratch_bytes) return fail(RTAMS_EINVAL, "overflow_bytes exceeds scratch_bytes");
  if (cfg->overflow_chunks < 0 || cfg->overflow_chunks > kMaxOverflowChunks)
    return fail(RTAMS_EINVAL, "overflow_chunks must be in 0..%d", kMaxOverflowChunks);
  size_t slice = (cfg->scratch_bytes - cfg->overflow_bytes) / (size_t)cfg->n_resources / kAlign * kAlign;
  if (slice < SL.fixed + kAlign)
    return fail(RTAMS_EINVAL, "scratch slice of %zu bytes is smaller than its fixed part %zu", slice,
                SL.fixed + kAlign);

  rtams_index *ix = new (std::nothrow) rtams_index();
  if (!ix) return fail(RTAMS_EINVAL, "out of host memory");
  ix->cfg = *cfg;
  ix->lay = L;
  char *base = static_cast<char *>(cfg->d_pool);
  Dev &D = ix->dev;
  D.d = cfg->d; D.nlist = cfg->nlist; D.metric = cfg->metric; D.T_m = cfg->block_vecs;
  D.d4 = cfg->d / 4;
  D.storage = cfg->storage;
  D.vchunks = cfg->storage == RTAMS_F16 ? cfg->d / 8 : cfg->storage == RTAMS_U8 ? cfg->d / 16 : cfg->d / 4;
  D.groups_per_block = cfg->block_vecs / kWave;
  D.nblocks = (uint32_t)L.nblocks;
  D.slab_cap = (uint32_t)(L.slab_cap > 0xffffffffull ? 0xffffffffull : L.slab_cap);
  D.T_mp = cfg->rearrange_threshold;
  D.block_stride = L.block_stride;
  D.ids_off = L.ids_off; D.vec_off = L.vec_off;
  D.blocks = base + L.blocks;
  D.ctrl = reinterpret_cast<Ctrl *>(base + L.ctrl);
  D.centroids = reinterpret_cast<float *>(base + L.centroids);
  D.centroids_t = reinterpret_cast<float *>(base + L.centroids_t);
  D.cnorm = reinterpret_cast<float *>(base + L.cnorm);
  D.csplit = reinterpret_cast<u32x4 *>(base + L.csplit);
  D.dgroups = (cfg->d + 31) / 32 * 4;
  D.codebooks = reinterpret_cast<float *>(base + L.codebooks);
  D.codebooks_t = reinterpret_cast<float *>(base + L.codebooks_t);
  D.pq_m = cfg->pq_m;
  D.reserved_len = reinterpret_cast<uint32_t *>(base + L.reserved_len);
  D.visible_len = reinterpret_cast<uint32_t *>(base + L.visible_len);
  D.online = reinterpret_cast<uint32_t *>(base + L.online);
  D.nblk = reinterpret_cast<uint32_t *>(base + L.nblk);
  D.exceed = reinterpret_cast<uint8_t *>(base + L.exceed);
  D.seg_dir = reinterpret_cast<int32_t *>(base + L.seg_dir);
  D.slab = reinterpret_cast<int32_t *>(base + L.slab);
  D.free_stack = reinterpret_cast<int32_t *>(base + L.free_stack);
  D.mark = reinterpret_cast<int32_t *>(base + L.mark);
  ix->hook = base + L.hook;
  ix->ins.assign = reinterpret_cast<int32_t *>(base + L.ins_assign);
  ix->ins.did = reinterpret_cast<uint32_t *>(base + L.ins_did);
  ix->ins.pscore = reinterpret_cast<double *>(base + L.ins_pscore);
  ix->ins.pidx = reinterpret_cast<int32_t *>(base + L.ins_pidx);
  ix->ins.part_cap = L.part_cap;
  ix->ins.tiles.tiles = (cfg->nlist + 127) / 128;
  ix->ins.tiles.tmin = reinterpret_cast<float *>(base + L.tc_min);
  ix->ins.tiles.cnt = reinterpret_cast<uint32_t *>(base + L.tc_cnt);
  ix->ins.tiles.col = reinterpret_cast<int32_t *>(base + L.tc_col);
  ix->ins.tiles.val = reinterpret_cast<float *>(base + L.tc_val);
  ix->ins.tile_rows = (int64_t)L.tile_rows;
  ix->ins.ysplit = reinterpret_cast<u32x4 *>(base + L.ins_ysplit);
  ix->ins.ynorm = reinterpret_cast<float *>(base + L.ins_ynorm);
  {
    uint32_t *a = reinterpret_cast<uint32_t *>(base + L.rearr_arrays);
    RearrangeScratch &R = ix->rearr;
    R.head = reinterpret_cast<RearrangeHead *>(base + L.rearr_head);
    R.cap = kRearrangeCap;
    R.mv_t = a; R.kind = a + kRearrangeCap; R.vic_rank = a + 2 * kRearrangeCap;
    R.vic_new = a + 3 * kRearrangeCap; R.old_src = a + 4 * kRearrangeCap;
    R.vic_list = reinterpret_cast<int32_t *>(a + 5 * kRearrangeCap);
    R.vic_seq = reinterpret_cast<int32_t *>(a + 6 * kRearrangeCap);
  }
  ix->avail_lb = L.nblocks;

  auto bail = [&](int code) { rtams_destroy(ix); return code; };
  // control data: everything in front of the blocks starts at zero, table directory at -1
  if (hipMemset(base, 0, L.blocks) != hipSuccess) return bail(fail(RTAMS_EHIP, "hipMemset of control data failed"));
  if (hipMemset(D.seg_dir, 0xff, (size_t)cfg->nlist * kTableSegs * 4) != hipSuccess)
    return bail(fail(RTAMS_EHIP, "hipMemset of the table directory failed"));
  void *hm = nullptr;
  if (hipHostMalloc(&hm, sizeof(HostMirror), hipHostMallocMapped) != hipSuccess)
    return bail(fail(RTAMS_EHIP, "hipHostMalloc failed"));
  ix->mirror = static_cast<HostMirror *>(hm);
  memset(hm, 0, sizeof(HostMirror));
  void *dm = nullptr;
  if (hipHostGetDevicePointer(&dm, hm, 0) != hipSuccess) return bail(fail(RTAMS_EHIP, "hipHostGetDevicePointer failed"));
  D.mirror = static_cast<HostMirror *>(dm);
  if (hipEventCreateWithFlags(&ix->data_done, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ix->fence_ev[0], hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ix->fence_ev[1], hipEventDisableTiming) != hipSuccess)
    return bail(fail(RTAMS_EHIP, "hipEventCreate failed"));

  ix->res = new (std::nothrow) Resource[cfg->n_resources + 1];
  if (!ix->res) return bail(fail(RTAMS_EINVAL, "out of host memory"));
  ix->n_res = cfg->n_resources;
  char *sb = static_cast<char *>(cfg->d_scratch);
  // the shared reserve behind the slices: the lease words (256 bytes), then two arrays of equal length,
  // each cut into overflow_chunks chunks
  char *ovf = sb + (size_t)cfg->n_resources * slice;
  const uint32_t ovf_chunks = cfg->overflow_bytes > 0 ? (uint32_t)(cfg->overflow_chunks > 0 ? cfg->overflow_chunks : 4) : 0u;
  const size_t ovf_bytes = ovf_chunks ? cfg->scratch_bytes - (size_t)cfg->n_resources * slice : 0;
  // entries per chunk: what is left after the lease words, over two arrays and the chunks, in whole 256-byte units
  const unsigned long long ovf_chunk_cap =
      ovf_bytes > kAlign ? (ovf_bytes - kAlign) / (2 * kAlign * ovf_chunks) * (kAlign / 4) : 0;
  if (ovf_chunks && ovf_chunk_cap == 0)
    return bail(fail(RTAMS_EINVAL, "overflow_bytes %zu holds no chunk (%u chunks asked for)", cfg->overflow_bytes, ovf_chunks));
  if (ovf_chunks && hipMemset(ovf, 0, kAlign) != hipSuccess) return bail(fail(RTAMS_EHIP, "hipMemset of the scratch reserve failed"));
  ix->ovf_leased = ovf_chunks ? reinterpret_cast<uint32_t *>(ovf) : nullptr;
  ix->ovf_chunks = ovf_chunks;
  ix->ovf_chunk_cap = ovf_chunk_cap;
  auto lay_slice = [&](Resource &R, char *p, const ScratchLayout &SL, size_t slice_bytes, bool with_reserve) -> int {
    SearchScratch &S = R.s;
    S.scores = reinterpret_cast<double *>(p + SL.scores);
    S.approx = reinterpret_cast<float *>(p + SL.approx);
    S.lut = reinterpret_cast<float *>(p + SL.lut);
    S.probe_list = reinterpret_cast<int32_t *>(p + SL.probe_list);
    S.probe_len = reinterpret_cast<uint32_t *>(p + SL.probe_len);
    S.qbase = reinterpret_cast<unsigned long long *>(p + SL.qbase);
    S.qtotal = reinterpret_cast<uint32_t *>(p + SL.qtotal);
    S.bound = reinterpret_cast<uint32_t *>(p + SL.bound);
    S.qnorm = reinterpret_cast<float *>(p + SL.qnorm);
    S.qsplit = reinterpret_cast<u32x4 *>(p + SL.qsplit);
    S.rec_cnt = reinterpret_cast<uint32_t *>(p + SL.rec_cnt);
    S.cursor = reinterpret_cast<unsigned long long *>(p + SL.cursor);
    S.list_cnt = reinterpret_cast<uint32_t *>(p + SL.list_cnt);
    S.pair_start = reinterpret_cast<uint32_t *>(p + SL.pair_start);
    S.pair_slot = reinterpret_cast<uint32_t *>(p + SL.pair_slot);
    S.grouped = reinterpret_cast<uint32_t *>(p + SL.grouped);
    S.plist = reinterpret_cast<uint4 *>(p + SL.plist);
    S.pistart = reinterpret_cast<uint32_t *>(p + SL.pistart);
    S.tile_desc = reinterpret_cast<uint4 *>(p + SL.tile_desc);
    S.item_cap = (uint32_t)SL.item_cap;
    S.queues = reinterpret_cast<ScanQueues *>(p + SL.queues);
    // the rest of the slice: two arrays of equal length
    S.cand_cap = (slice_bytes - SL.fixed) / (2 * kAlign) * (kAlign / 4);
    S.rec_key = reinterpret_cast<uint32_t *>(p + SL.records);
    S.rec_pos = S.rec_key + S.cand_cap;
    S.ovf_leased = with_reserve ? ix->ovf_leased : nullptr;
    S.ovf_chunks = with_reserve ? ovf_chunks : 0u;
    S.ovf_chunk_cap = with_reserve ? ovf_chunk_cap : 0ull;
    S.ovf_key = reinterpret_cast<uint32_t *>(ovf + kAlign);
    S.ovf_pos = S.ovf_key + ovf_chunk_cap * ovf_chunks;
    S.req_chunk = reinterpret_cast<uint32_t *>(p + SL.req_words);
    S.req_done = S.req_chunk + 1;
    S.req_cursor = reinterpret_cast<unsigned long long *>(p + SL.req_words + 8);
    if (hipMemset(p + SL.req_words, 0, 16) != hipSuccess) return fail(RTAMS_EHIP, "hipMemset of the scratch failed");
    if (hipEventCreateWithFlags(&R.done, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&R.scan_done, hipEventDisableTiming) != hipSuccess ||
        hipEventCreate(&R.t0) != hipSuccess || hipEventCreate(&R.t1) != hipSuccess)
      return fail(RTAMS_EHIP, "hipEventCreate failed");
    return RTAMS_OK;
  };
  for (int r = 0; r < ix->n_res; ++r) {
    const int rc = lay_slice(ix->res[r], sb + (size_t)r * slice, SL, slice, true);
    if (rc) return bail(rc);
  }
  // the extra resource over the library's static array, for requests of up to kStaticMaxBatch queries
  // (its fixed part is laid out for that many; an index whose fixed part alone does not fit goes without)
  {
    rtams_config small = *cfg;
    small.max_batch = cfg->max_batch < kStaticMaxBatch ? cfg->max_batch : kStaticMaxBatch;
    ScratchLayout SS;
    lay_out_scratch(&small, &SS);
    void *sp = nullptr;
    const int rc = static_scratch_of_current_device(&sp);
    if (rc) return bail(rc);
    ix->static_max_batch = small.max_batch;
    ix->static_ok = SS.fixed + 64 * kAlign <= kStaticScratchBytes;
    if (ix->static_ok) {
      const int rc2 = lay_slice(ix->res[ix->n_res], static_cast<char *>(sp), SS, kStaticScratchBytes, false);
      if (rc2) return bail(rc2);
    }
  }
  if (hipDeviceSynchronize() != hipSuccess) return bail(fail(RTAMS_EHIP, "hipDeviceSynchronize failed"));
  *out = ix;
  return RTAMS_OK;
}

int rtams_destroy(rtams_index *ix) {
  if (!ix) return RTAMS_OK;
  if (ix->have_data_stream) (void)hipStreamSynchronize(ix->data_stream);
  for (int r = 0; ix->res && r <= ix->n_res; ++r)
    if (ix->res[r].done) {
      (void)hipEventSynchronize(ix->res[r].done);
      (void)hipEventDestroy(ix->res[r].done);
      if (ix->res[r].t0) (void)hipEventDestroy(ix->res[r].t0);
      if (ix->res[r].t1) (void)hipEventDestroy(ix->res[r].t1);
      if (ix->res[r].scan_done) (void)hipEventDestroy(ix->res[r].scan_done);
    }
  delete[] ix->res;
  if (ix->data_done) (void)hipEventDestroy(ix->data_done);
  for (hipEvent_t e : ix->fence_ev)
    if (e) (void)hipEventDestroy(e);
  if (ix->mirror) (void)hipHostFree((void *)ix->mirror);
  delete ix;
  return RTAMS_OK;
}

int rtams_set_centroids(rtams_index *ix, const float *d_centroids, void *hip_stream) {
  if (!ix || !d_centroids) return fail(RTAMS_EINVAL, "NULL argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  if (ix->ntotal_host > 0) return fail(RTAMS_ESTATE, "centroids cannot change once vectors are in");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int rc = enter_data_stream(ix, s);
  if (rc) return rc;
  DataStreamScope scope{ix, s};
  HIP_TRY(hipMemcpyAsync(ix->dev.centroids, d_centroids, (size_t)ix->cfg.nlist * ix->cfg.d * 4,
                         hipMemcpyDeviceToDevice, s));
  launch_centroid_norms(ix->dev, s);
  launch_centroid_transpose(ix->dev, s);
  HIP_TRY(hipGetLastError());
  ix->has_centroids = true;
  return RTAMS_OK;
}

int rtams_set_codebooks(rtams_index *ix, const float *d_codebooks, void *hip_stream) {
  if (!ix || !d_codebooks) return fail(RTAMS_EINVAL, "NULL argument");
  if (ix->cfg.pq_m == 0) return fail(RTAMS_ESTATE, "the index holds flat lists (pq_m is 0)");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  if (ix->ntotal_host > 0) return fail(RTAMS_ESTATE, "codebooks cannot change once vectors are in");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int rc = enter_data_stream(ix, s);
  if (rc) return rc;
  DataStreamScope scope{ix, s};
  HIP_TRY(hipMemcpyAsync(ix->dev.codebooks, d_codebooks, (size_t)256 * ix->cfg.d * 4, hipMemcpyDeviceToDevice, s));
  launch_pq_transpose(ix->dev, s);
  HIP_TRY(hipGetLastError());
  ix->has_codebooks = true;
  return RTAMS_OK;
}

int rtams_add(rtams_index *ix, int64_t n, const float *d_vecs, const int64_t *d_ids, void *hip_stream) {
  if (!ix || n < 0 || (n > 0 && !d_vecs)) return fail(RTAMS_EINVAL, "bad argument to add");
  if (!ix->has_centroids) return fail(RTAMS_ESTATE, "add before set_centroids");
  if (ix->cfg.pq_m > 0 && !ix->has_codebooks) return fail(RTAMS_ESTATE, "add before set_codebooks");
  if (n == 0) return RTAMS_OK;
  std::lock_guard<std::mutex> g(ix->data_mutex);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const Dev &D = ix->dev;
  if (ix->mirror->error == RTAMS_EPOOL) return fail(RTAMS_EPOOL, "the pool overflowed earlier; index is read-only");

  // Upper bound of the blocks this batch can open: one partly filled block per
  // touched list plus the full ones.
  int64_t need = (n < D.nlist ? n : D.nlist) + n / D.T_m;
  if (need > ix->avail_lb || ix->pending_adds.size() >= 4096) tighten_pool_bound(ix);
  if (need > ix->avail_lb) {  // what the device has reported does not do: wait for it and read its counters
    int rc = sync_data(ix);
    if (rc) return rc;
    Ctrl c;
    if ((rc = read_ctrl(ix, &c))) return rc;
    ++ix->add_waits;
    ix->pending_adds.clear();
    ix->pending_need = 0;
    ix->avail_lb = (int64_t)D.nblocks - (int64_t)c.cur_P + (c.free_top > 0 ? c.free_top : 0);
    if (need > ix->avail_lb)
      return fail(RTAMS_EPOOL, "add of %lld vectors may need %lld blocks, %lld left in the pool",
                  (long long)n, (long long)need, (long long)ix->avail_lb);
  }
  int rc = enter_data_stream(ix, s);
  if (rc) return rc;
  DataStreamScope scope{ix, s};
  const int64_t round = ix->cfg.max_add_batch;
  const bool ordered = ix->ordered_add.load(std::memory_order_relaxed) != 0;
  const uint32_t seq = ++ix->add_seq;
  for (int64_t o = 0; o < n; o += round) {
    int64_t m = n - o < round ? n - o : round;
    const float *Y = d_vecs + (size_t)o * D.d;
    if (ordered) {
      assign_round(ix, m, Y, false, ix->ins.assign, s);
      launch_reserve_ordered(D, m, ix->ins, s);
    } else {
      assign_round(ix, m, Y, true, ix->ins.assign, s);
    }
    launch_open(D, s);
    if (D.pq_m > 0) launch_pq_fill(D, m, Y, d_ids ? d_ids + o : nullptr, ix->ntotal_host + o, ix->ins, s);
    else launch_fill(D, m, Y, d_ids ? d_ids + o : nullptr, ix->ntotal_host + o, ix->ins, s);
    // only its last round completes the call: the rounds before it report under the call before
    launch_publish(D, o + round >= n ? seq : seq - 1u, s);
  }
  HIP_TRY(hipGetLastError());
  ix->avail_lb -= need;
  ix->pending_adds.push_back({seq, need});
  ix->pending_need += need;
  ix->ntotal_host += n;
  // Exceed() held for some list when an earlier batch was published (the device
  // reports it through pinned memory): one rearrangement round behind this batch
  if (ix->cfg.rearrange_threshold > 0 && ix->mirror->exceed_lists > 0) {
    if ((rc = rearrange_round(ix, -1, s))) return rc;
  }
  return RTAMS_OK;
}

// What rtams_search and rtams_search_noalloc share: the argument checks, and the request itself on the
// resource the caller took (pooled: a slice of the caller's scratch; n_res: the library's static array).
static int check_search_args(rtams_index *ix, int64_t nq, const float *d_queries, int32_t k, int32_t nprobe,
                             float *d_out_dist, int64_t *d_out_ids) {
  if (!ix || nq < 0) return fail(RTAMS_EINVAL, "bad argument to search");
  if (nq > ix->cfg.max_batch) return fail(RTAMS_EINVAL, "nq %lld exceeds max_batch %d", (long long)nq, ix->cfg.max_batch);
  if (k < 1 || k > ix->cfg.max_k) return fail(RTAMS_EINVAL, "k %d outside 1..max_k %d", k, ix->cfg.max_k);
  if (nprobe < 1 || nprobe > ix->cfg.max_nprobe)
    return fail(RTAMS_EINVAL, "nprobe %d outside 1..max_nprobe %d", nprobe, ix->cfg.max_nprobe);
  if (!ix->has_centroids) return fail(RTAMS_ESTATE, "search before set_centroids");
  if (ix->cfg.pq_m > 0 && !ix->has_codebooks) return fail(RTAMS_ESTATE, "search before set_codebooks");
  if (nq > 0 && (!d_queries || !d_out_dist || !d_out_ids)) return fail(RTAMS_EINVAL, "NULL buffer");
  return RTAMS_OK;
}

static int search_on(rtams_index *ix, int r, int64_t nq, const float *d_queries, int32_t k, int32_t nprobe,
                     float *d_out_dist, int64_t *d_out_ids, void *hip_stream) {
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Dev D = ix->dev;
  {  // flat float lists: requests whose tiles hold several queries scan on the matrix cores (0 never, 1 by the rule below, 2 always)
    const int64_t mode = ix->scan_mfma.load(std::memory_order_relaxed);
    // A tile is the queries of the request that probe one list.  With at least as many (query, list)
    // pairs as lists, or with a list far longer than the average (a hot list is probed by a good
    // share of any batch and holds most of the bytes), tiles of several queries do most of the work:
    // that is what the matrix-core kernel is for.  A request whose pairs spread thinly over many lists
    // of similar length has tiles of one query each and is better off on the vector unit (measured:
    // 64 queries x 32 probes over 8,192 lists of 768 dimensions, 643 against 667 us).
    const int64_t avg_len = ix->ntotal_host / ix->cfg.nlist + 1;
    const bool shared = nq * nprobe >= ix->cfg.nlist || (int64_t)ix->mirror->max_len >= 16 * avg_len;
    D.scan_mfma = D.pq_m == 0 && D.storage == RTAMS_F32 &&
                  (mode == 2 || (mode == 1 && nq >= kMmMinBatch && shared));
  }
  D.scan_byte_weight = (int32_t)ix->scan_byte_weight.load(std::memory_order_relaxed);
  D.scan_min_choice = (int32_t)ix->scan_min_choice.load(std::memory_order_relaxed);
  // a long scan: its (query, list) pairs are expected to meet this many list bytes (lists of average length)
  const int64_t excl = ix->scan_exclusive_pairs.load(std::memory_order_relaxed);
  const int64_t vec_bytes = D.pq_m > 0 ? D.pq_m : (int64_t)D.vchunks * 16;
  const int64_t pair_bytes = nq * nprobe * (ix->ntotal_host / ix->cfg.nlist + 1) * vec_bytes;
  const bool long_scan = excl > 0 && nq * nprobe >= excl &&
                         pair_bytes >= ix->scan_exclusive_bytes.load(std::memory_order_relaxed);
  D.scan_steal = long_scan && ix->scan_steal.load(std::memory_order_relaxed) != 0;
  const SearchScratch &S = ix->res[r].s;
  // a rearrangement is switching block tables: start behind its last switch
  if (ix->fence_cur) (void)hipStreamWaitEvent(s, ix->fence_cur, 0);
  coarse_and_plan(ix, nq, d_queries, nprobe, S, nullptr, s);
  // The grouped scan is cut into work items of bounded size, one wavefront each;
  // the budget of items grows with the request so that a small batch still
  // spreads over the chip and a large one is not drowned in per-item overhead.
  int64_t budget = nq * nprobe * ix->scan_items_per_pair.load(std::memory_order_relaxed);
  const int64_t cap = ix->scan_max_items.load(std::memory_order_relaxed);
  if (budget > cap) budget = cap;
  if (budget < nq * nprobe) budget = nq * nprobe;  // a (query, list) pair is at least one item
  if (budget < 1024) budget = 1024;
  launch_group(D, nq, nprobe, ix->cfg.max_nprobe, k, d_queries, (int)budget, S, s);
  const bool timed = ix->profile_scan.load(std::memory_order_relaxed) != 0;
  if (timed) ix->timed_scans[D.pq_m > 0 ? 2 : D.scan_mfma ? 1 : 0].fetch_add(1, std::memory_order_relaxed);
  if (long_scan) {  // behind the long scan enqueued before it
    std::lock_guard<std::mutex> chain(ix->scan_mutex);
    if (ix->scan_tail && ix->scan_tail != ix->res[r].scan_done) (void)hipStreamWaitEvent(s, ix->scan_tail, 0);
    if (timed) (void)hipEventRecord(ix->res[r].t0, s);
    launch_scan(D, nq, nprobe, ix->cfg.max_nprobe, d_queries, (int)budget, S, s);
    if (timed) { (void)hipEventRecord(ix->res[r].t1, s); ix->res[r].timed = true; }
    (void)hipEventRecord(ix->res[r].scan_done, s);
    ix->scan_tail = ix->res[r].scan_done;
  } else {
    if (timed) (void)hipEventRecord(ix->res[r].t0, s);
    launch_scan(D, nq, nprobe, ix->cfg.max_nprobe, d_queries, (int)budget, S, s);
    if (timed) { (void)hipEventRecord(ix->res[r].t1, s); ix->res[r].timed = true; }
  }
  launch_select(D, nq, k, nprobe, ix->cfg.max_nprobe, d_queries, S, d_out_dist, d_out_ids, s);
  hipError_t e = hipGetLastError();
  hipError_t e2 = hipEventRecord(ix->res[r].done, s);
  ix->res[r].state.store(RES_PENDING, std::memory_order_release);
  if (e != hipSuccess || e2 != hipSuccess)
    return fail(RTAMS_EHIP, "search launch failed: %s", hipGetErrorString(e != hipSuccess ? e : e2));
  return RTAMS_OK;
}

int rtams_search(rtams_index *ix, int64_t nq, const float *d_queries, int32_t k, int32_t nprobe,
                 float *d_out_dist, int64_t *d_out_ids, void *hip_stream) {
  const int rc = check_search_args(ix, nq, d_queries, k, nprobe, d_out_dist, d_out_ids);
  if (rc || nq == 0) return rc;
  std::shared_lock<std::shared_mutex> in_flight(ix->fence_mutex);
  const int r = acquire(ix);
  if (r < 0) return fail(RTAMS_EBUSY, "all %d stream resources are in flight", ix->n_res);
  return search_on(ix, r, nq, d_queries, k, nprobe, d_out_dist, d_out_ids, hip_stream);
}

int rtams_search_noalloc(rtams_index *ix, int64_t nq, const float *d_queries, int32_t k, int32_t nprobe,
                         float *d_out_dist, int64_t *d_out_ids, void *hip_stream) {
  const int rc = check_search_args(ix, nq, d_queries, k, nprobe, d_out_dist, d_out_ids);
  if (rc || nq == 0) return rc;
  if (nq > kStaticMaxBatch)
    return fail(RTAMS_EINVAL, "nq %lld exceeds the %d queries a request on the library's static scratch may hold",
                (long long)nq, kStaticMaxBatch);
  if (!ix->static_ok)
    return fail(RTAMS_EINVAL, "the fixed part of a request of this index (nlist %d, max_nprobe %d) does not fit the "
                              "library's static scratch of %zu bytes", ix->cfg.nlist, ix->cfg.max_nprobe, kStaticScratchBytes);
  std::shared_lock<std::shared_mutex> in_flight(ix->fence_mutex);
  // the one resource over the static array: free, or its last request has finished
  Resource &R = ix->res[ix->n_res];
  int st = R.state.load(std::memory_order_acquire);
  bool mine = false;
  if (st == RES_FREE) mine = R.state.compare_exchange_strong(st, RES_BUSY, std::memory_order_acq_rel);
  else if (st == RES_PENDING && hipEventQuery(R.done) == hipSuccess)
    mine = R.state.compare_exchange_strong(st, RES_BUSY, std::memory_order_acq_rel);
  (void)hipGetLastError();  // hipEventQuery leaves hipErrorNotReady behind
  if (!mine) return fail(RTAMS_EBUSY, "the request before this one on the static scratch has not finished");
  harvest(ix, R);
  return search_on(ix, ix->n_res, nq, d_queries, k, nprobe, d_out_dist, d_out_ids, hip_stream);
}

// Grace period: the work enqueued next on the data stream starts only after
// every search request that is in flight now has finished, and every search
// enqueued from now on starts behind `ev` (the table switch just enqueued).
static int fence_searches(rtams_index *ix, hipEvent_t ev, hipStream_t s) {
  HIP_TRY(hipEventRecord(ev, s));
  std::unique_lock<std::shared_mutex> g(ix->fence_mutex);
  ix->fence_cur = ev;
  for (int r = 0; r <= ix->n_res; ++r)  // the pooled resources and the one over the static array
    if (ix->res[r].state.load(std::memory_order_acquire) == RES_PENDING)
      HIP_TRY(hipStreamWaitEvent(s, ix->res[r].done, 0));
  return RTAMS_OK;
}

static int rearrange_round(rtams_index *ix, int32_t list, hipStream_t s) {
  const Dev &D = ix->dev;
  launch_rearr_plan(D, ix->rearr, list, s);
  launch_rearr_step(D, ix->rearr, 1, s);   // occupants out of the way, their tables switched
  int rc = fence_searches(ix, ix->fence_ev[0], s);
  if (rc) return rc;
  launch_rearr_step(D, ix->rearr, 2, s);   // the list's blocks into place, its table switched
  if ((rc = fence_searches(ix, ix->fence_ev[1], s))) return rc;
  launch_rearr_release(D, ix->rearr, s);
  HIP_TRY(hipGetLastError());
  return RTAMS_OK;
}

int rtams_rearrange(rtams_index *ix, int32_t list, void *hip_stream) {
  if (!ix || list < -1 || list >= ix->cfg.nlist) return fail(RTAMS_EINVAL, "bad list");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int rc = enter_data_stream(ix, s);
  if (rc) return rc;
  DataStreamScope scope{ix, s};
  // A round moves at most kRearrangeCap blocks, and no more than the pool has spare blocks for; only the
  // device knows whether another is owed, so every round is waited for.
  const int64_t max_rounds = (int64_t)ix->dev.nblocks + 8 * (int64_t)ix->cfg.nlist + 64;
  if (list >= 0) {
    for (int64_t it = 0; it < max_rounds; ++it) {
      if ((rc = rearrange_round(ix, list, s))) return rc;  // blocks in use are the same before and after
      HIP_TRY(hipStreamSynchronize(s));
      const uint32_t state = ix->mirror->rearr_state;
      if (state == 2)
        return fail(RTAMS_ENOSPARE, "list %d: no spare block in the pool to move a block through; its chain is as it was", list);
      if (state == 0) break;
    }
    return RTAMS_OK;
  }
  // Every list for which Exceed() holds, one after the other.  A list that stalls for lack of a spare
  // block keeps its flag; when a whole turn through the exceeding lists moved nothing, the call gives up.
  int64_t stalled_in_a_row = 0;
  for (int64_t it = 0; it < max_rounds; ++it) {
    if (ix->mirror->exceed_lists == 0) break;
    if ((rc = rearrange_round(ix, -1, s))) return rc;
    HIP_TRY(hipStreamSynchronize(s));
    if (ix->mirror->rearr_state == 2) {
      if (++stalled_in_a_row >= (int64_t)ix->mirror->exceed_lists)
        return fail(RTAMS_ENOSPARE, "%u lists exceed, and the pool has no spare block to move a block through",
                    ix->mirror->exceed_lists);
    } else {
      stalled_in_a_row = 0;
    }
  }
  return RTAMS_OK;
}

int rtams_probe(rtams_index *ix, int64_t nq, const float *d_queries, int32_t nprobe, int32_t *d_out,
                void *hip_stream) {
  if (!ix || nq < 0 || nq > ix->cfg.max_batch || nprobe < 1 || nprobe > ix->cfg.max_nprobe)
    return fail(RTAMS_EINVAL, "bad argument to probe");
  if (!ix->has_centroids) return fail(RTAMS_ESTATE, "probe before set_centroids");
  if (nq == 0) return RTAMS_OK;
  if (!d_queries || !d_out) return fail(RTAMS_EINVAL, "NULL buffer");
  std::shared_lock<std::shared_mutex> in_flight(ix->fence_mutex);
  int r = acquire(ix);
  if (r < 0) return fail(RTAMS_EBUSY, "all %d stream resources are in flight", ix->n_res);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const SearchScratch &S = ix->res[r].s;
  coarse_and_plan(ix, nq, d_queries, nprobe, S, d_out, s);
  hipError_t e = hipGetLastError();
  hipError_t e2 = hipEventRecord(ix->res[r].done, s);
  ix->res[r].state.store(RES_PENDING, std::memory_order_release);
  if (e != hipSuccess || e2 != hipSuccess) return fail(RTAMS_EHIP, "probe launch failed");
  return RTAMS_OK;
}

int rtams_assign(rtams_index *ix, int64_t n, const float *d_vecs, int32_t *d_out, void *hip_stream) {
  if (!ix || n < 0) return fail(RTAMS_EINVAL, "bad argument to assign");
  if (!ix->has_centroids) return fail(RTAMS_ESTATE, "assign before set_centroids");
  if (n == 0) return RTAMS_OK;
  if (!d_vecs || !d_out) return fail(RTAMS_EINVAL, "NULL buffer");
  std::lock_guard<std::mutex> g(ix->data_mutex);  // shares the insertion scratch
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int rc = enter_data_stream(ix, s);
  if (rc) return rc;
  DataStreamScope scope{ix, s};
  const int64_t round = ix->cfg.max_add_batch;
  for (int64_t o = 0; o < n; o += round) {
    int64_t m = n - o < round ? n - o : round;
    assign_round(ix, m, d_vecs + (size_t)o * ix->dev.d, false, d_out + o, s);
  }
  HIP_TRY(hipGetLastError());
  return RTAMS_OK;
}

// ------------------------------------------------------------ introspection

int rtams_ntotal(rtams_index *ix, int64_t *out) {
  if (!ix || !out) return fail(RTAMS_EINVAL, "NULL argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  Ctrl c;
  if ((rc = read_ctrl(ix, &c))) return rc;
  *out = (int64_t)c.ntotal;
  return RTAMS_OK;
}

int rtams_list_sizes(rtams_index *ix, int64_t *out) {
  if (!ix || !out) return fail(RTAMS_EINVAL, "NULL argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  uint32_t *tmp = new (std::nothrow) uint32_t[ix->cfg.nlist];
  if (!tmp) return fail(RTAMS_EINVAL, "out of host memory");
  hipError_t e = hipMemcpy(tmp, ix->dev.visible_len, (size_t)ix->cfg.nlist * 4, hipMemcpyDeviceToHost);
  for (int k = 0; k < ix->cfg.nlist; ++k) out[k] = tmp[k];
  delete[] tmp;
  if (e != hipSuccess) return fail(RTAMS_EHIP, "hipMemcpy failed: %s", hipGetErrorString(e));
  return RTAMS_OK;
}

int rtams_list_size(rtams_index *ix, int32_t list, int64_t *out) {
  if (!ix || !out || list < 0 || list >= ix->cfg.nlist) return fail(RTAMS_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  uint32_t v = 0;
  HIP_TRY(hipMemcpy(&v, ix->dev.visible_len + list, 4, hipMemcpyDeviceToHost));
  *out = v;
  return RTAMS_OK;
}

int rtams_list_info(rtams_index *ix, int32_t list, int64_t *blocks, int64_t *runs, int64_t *online) {
  if (!ix || list < 0 || list >= ix->cfg.nlist) return fail(RTAMS_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  int32_t *d4 = reinterpret_cast<int32_t *>(ix->hook);
  launch_list_info(ix->dev, list, d4, nullptr);
  int32_t h[4];
  HIP_TRY(hipMemcpy(h, d4, sizeof(h), hipMemcpyDeviceToHost));
  if (blocks) *blocks = h[0];
  if (runs) *runs = h[1];
  if (online) *online = h[2];
  return RTAMS_OK;
}

int rtams_list_export(rtams_index *ix, int32_t list, int64_t cap, int64_t *d_ids, float *d_vecs,
                      int64_t *n_out, void *hip_stream) {
  if (!ix || list < 0 || list >= ix->cfg.nlist || cap < 0) return fail(RTAMS_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  uint32_t len = 0;
  HIP_TRY(hipMemcpy(&len, ix->dev.visible_len + list, 4, hipMemcpyDeviceToHost));
  if (n_out) *n_out = len;
  if ((int64_t)len > cap) return fail(RTAMS_EINVAL, "list %d holds %u vectors, cap is %lld", list, len, (long long)cap);
  if (ix->cfg.pq_m > 0 && d_vecs) return fail(RTAMS_ESTATE, "the lists hold codes: use rtams_list_export_codes");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  launch_export(ix->dev, list, len, d_ids, d_vecs, s);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(s));
  return RTAMS_OK;
}

int rtams_list_export_codes(rtams_index *ix, int32_t list, int64_t cap, int64_t *d_ids, uint8_t *d_codes,
                            int64_t *n_out, void *hip_stream) {
  if (!ix || list < 0 || list >= ix->cfg.nlist || cap < 0) return fail(RTAMS_EINVAL, "bad argument");
  if (ix->cfg.pq_m == 0) return fail(RTAMS_ESTATE, "the index holds flat lists (pq_m is 0)");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  uint32_t len = 0;
  HIP_TRY(hipMemcpy(&len, ix->dev.visible_len + list, 4, hipMemcpyDeviceToHost));
  if (n_out) *n_out = len;
  if ((int64_t)len > cap) return fail(RTAMS_EINVAL, "list %d holds %u vectors, cap is %lld", list, len, (long long)cap);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  launch_pq_export(ix->dev, list, len, d_ids, d_codes, s);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(s));
  return RTAMS_OK;
}

int rtams_list_chain(rtams_index *ix, int32_t list, int64_t cap, int32_t *chain, int64_t *n_out) {
  if (!ix || list < 0 || list >= ix->cfg.nlist || cap < 0) return fail(RTAMS_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  uint32_t nb = 0;
  HIP_TRY(hipMemcpy(&nb, ix->dev.nblk + list, 4, hipMemcpyDeviceToHost));
  if (n_out) *n_out = nb;
  if ((int64_t)nb > cap) return fail(RTAMS_EINVAL, "chain of %u blocks, cap is %lld", nb, (long long)cap);
  if (nb == 0) return RTAMS_OK;
  if (!chain) return fail(RTAMS_EINVAL, "NULL chain");
  launch_chain_copy(ix->dev, list, ix->dev.mark, nullptr);  // the validation marks double as staging
  HIP_TRY(hipMemcpy(chain, ix->dev.mark, (size_t)nb * 4, hipMemcpyDeviceToHost));
  return RTAMS_OK;
}

int rtams_pool_stats(rtams_index *ix, rtams_stats *out) {
  if (!ix || !out) return fail(RTAMS_EINVAL, "NULL argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  Ctrl c;
  if ((rc = read_ctrl(ix, &c))) return rc;
  memset(out, 0, sizeof(*out));
  out->ntotal = (int64_t)c.ntotal;
  out->blocks_total = ix->dev.nblocks;
  out->blocks_handed_out = c.cur_P;
  out->blocks_free = c.free_top > 0 ? c.free_top : 0;
  out->blocks_in_use = out->blocks_handed_out - out->blocks_free;
  out->block_bytes = (int64_t)ix->lay.block_stride;
  out->pool_bytes = (int64_t)ix->cfg.pool_bytes;
  out->meta_bytes = (int64_t)ix->lay.blocks;
  out->utilisation = (double)out->blocks_in_use / (double)out->blocks_total;
  out->lists_exceeding = c.exceed_lists;
  out->table_entries_used = c.slab_cur;
  out->table_entries_total = (int64_t)ix->lay.slab_cap;
  out->overflow_chunks = ix->ovf_chunks;
  out->overflow_chunk_entries = (int64_t)ix->ovf_chunk_cap;
  out->rearrangement_state = ix->mirror->rearr_state;
  if (ix->ovf_leased) {  // as of now: searches in flight on other streams may hold chunks
    uint32_t leased[kMaxOverflowChunks];
    HIP_TRY(hipMemcpy(leased, ix->ovf_leased, sizeof(uint32_t) * ix->ovf_chunks, hipMemcpyDeviceToHost));
    for (uint32_t e = 0; e < ix->ovf_chunks; ++e) out->overflow_chunks_leased += leased[e] != 0;
  }
  out->add_waits = ix->add_waits;
  ix->avail_lb = out->blocks_total - out->blocks_in_use;
  ix->pending_adds.clear();  // the data stream was waited for: every call is in those counters
  ix->pending_need = 0;
  return RTAMS_OK;
}

int rtams_validate(rtams_index *ix, void *hip_stream) {
  if (!ix) return fail(RTAMS_EINVAL, "NULL argument");
  std::lock_guard<std::mutex> g(ix->data_mutex);
  int rc = sync_data(ix);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int32_t *res = reinterpret_cast<int32_t *>(ix->hook + 64);
  launch_validate(ix->dev, res, s);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipStreamSynchronize(s));
  int32_t h[2];
  HIP_TRY(hipMemcpy(h, res, sizeof(h), hipMemcpyDeviceToHost));
  static const char *what[] = {"consistent", "reserved length differs from visible length",
                               "chain length is not ceil(len / T_m)", "table entry out of range",
                               "header owner/seq/capacity disagrees with the table",
                               "header prev/next disagrees with the table",
                               "header size disagrees with the list length", "block reachable twice",
                               "blocks in chains + free stack != cur_P", "sum of list lengths != ntotal"};
  if (h[0] != 0)
    return fail(RTAMS_EINVAL, "validate: %s (argument %d)", h[0] >= 1 && h[0] <= 9 ? what[h[0]] : "unknown", h[1]);
  return RTAMS_OK;
}

int rtams_poll_error(rtams_index *ix) {
  if (!ix) return RTAMS_EINVAL;
  const int32_t e = ix->mirror->error;  // the pool's state first: it is the one that stays
  return e ? e : ix->mirror->search_error;
}

int rtams_clear_error(rtams_index *ix) {
  if (!ix) return fail(RTAMS_EINVAL, "NULL argument");
  const int32_t zero = 0;
  HIP_TRY(hipMemcpy(&ix->dev.ctrl->search_error, &zero, sizeof(zero), hipMemcpyHostToDevice));
  ix->mirror->search_error = 0;
  return RTAMS_OK;
}

int rtams_scan_time(rtams_index *ix, double *ms_sum, int64_t *launches, int reset) {
  if (!ix) return fail(RTAMS_EINVAL, "NULL argument");
  for (int r = 0; r < ix->n_res; ++r) {  // collect from requests that have finished
    int st = RES_PENDING;
    if (ix->res[r].state.load(std::memory_order_acquire) == RES_PENDING &&
        hipEventQuery(ix->res[r].done) == hipSuccess &&
        ix->res[r].state.compare_exchange_strong(st, RES_BUSY, std::memory_order_acq_rel)) {
      harvest(ix, ix->res[r]);
      ix->res[r].state.store(RES_FREE, std::memory_order_release);
    }
  }
  (void)hipGetLastError();
  std::lock_guard<std::mutex> g(ix->prof_mutex);
  if (ms_sum) *ms_sum = ix->scan_ms;
  if (launches) *launches = ix->scan_launches;
  if (reset) { ix->scan_ms = 0.0; ix->scan_launches = 0; }
  return RTAMS_OK;
}

int rtams_scan_kernels(rtams_index *ix, int64_t *launches3, int reset) {
  if (!ix || !launches3) return fail(RTAMS_EINVAL, "NULL argument");
  for (int i = 0; i < 3; ++i)
    launches3[i] = reset ? ix->timed_scans[i].exchange(0, std::memory_order_relaxed)
                         : ix->timed_scans[i].load(std::memory_order_relaxed);
  return RTAMS_OK;
}

int rtams_copy_plain(void *d_dst, const void *d_src, size_t bytes, void *hip_stream) {
  if (!d_dst || !d_src || bytes % 16) return fail(RTAMS_EINVAL, "copy needs buffers and a multiple of 16 bytes");
  launch_copy_plain(d_dst, d_src, bytes, static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return RTAMS_OK;
}

int rtams_read_plain(const void *d_src, size_t bytes, float *d_sink, void *hip_stream) {
  if (!d_src || !d_sink || bytes % 16) return fail(RTAMS_EINVAL, "read needs buffers and a multiple of 16 bytes");
  launch_read_plain(d_src, bytes, d_sink, static_cast<hipStream_t>(hip_stream));
  HIP_TRY(hipGetLastError());
  return RTAMS_OK;
}

int rtams_set_param(rtams_index *ix, const char *key, int64_t value) {
  if (!ix || !key) return fail(RTAMS_EINVAL, "NULL argument");
  if (!strcmp(key, "profile_scan")) { ix->profile_scan = value; return RTAMS_OK; }
  if (!strcmp(key, "ordered_add")) { ix->ordered_add = value; return RTAMS_OK; }
  if (!strcmp(key, "use_mfma")) { ix->use_mfma = value; return RTAMS_OK; }
  if (!strcmp(key, "scan_mfma")) { ix->scan_mfma = value; return RTAMS_OK; }
  if (!strcmp(key, "scan_exclusive_pairs")) { ix->scan_exclusive_pairs = value > 0 ? value : 0; return RTAMS_OK; }
  if (!strcmp(key, "scan_steal")) { ix->scan_steal = value != 0; return RTAMS_OK; }
  if (!strcmp(key, "scan_exclusive_bytes")) { ix->scan_exclusive_bytes = value > 0 ? value : 0; return RTAMS_OK; }
  if (!strcmp(key, "scan_min_choice")) { ix->scan_min_choice = value < 0 ? -1 : value > 7 ? 7 : value; return RTAMS_OK; }
  if (!strcmp(key, "scan_byte_weight")) { ix->scan_byte_weight = value > 0 ? value : 0; return RTAMS_OK; }
  if (!strcmp(key, "scan_max_items")) { ix->scan_max_items = value > 1024 ? value : 1024; return RTAMS_OK; }
  if (!strcmp(key, "scan_items_per_pair")) { ix->scan_items_per_pair = value > 0 ? value : 1; return RTAMS_OK; }
  return fail(RTAMS_EINVAL, "unknown parameter %s", key);
}

}  // extern "C"
