// What a search request needs between its probe lists and its scan: the pruning bound of every
// query (from a sample of its nearest candidates), the (query, list) pairs grouped by list, and
// the scan's work items, cut and shared out over the XCDs.  One launch, three kinds of workgroup.
#include "search_common.h"

namespace rtams {

// ------------------------------------------------------------- pruning bound
constexpr int kSampleMax = 4096;  // candidates the bound of a query is taken from, at most
#ifndef RTAMS_SAMPLE_DIVISOR
#define RTAMS_SAMPLE_DIVISOR 4
#endif
constexpr int kSampleDivisor = RTAMS_SAMPLE_DIVISOR;
constexpr int kNoBoundBelow = 4096;  // candidates of a query up to which the scan keeps them all

// The scan writes nothing for a candidate that cannot be among the k best of
// its query: before it starts, every query gets a BOUND, the k-th best score
// of a sample of its candidates (the first few groups of its nearest probed
// lists, where most of its neighbours are).  The k-th best of any k or more
// candidates cannot be better than the final k-th best, so keeping what is not
// worse than the bound loses nothing.  One workgroup per query: a wavefront per
// group of 64 vectors, lane = vector, scores to LDS, radix selection there.
// These workgroups run beside the one that groups the pairs (same launch): both
// need only the plan, and the scan needs both.
// What the sample needs of the nearest list, read ahead by the caller (every one of these is a round
// trip to memory, and read where they are used they would follow one another): the list, its
// length, its number of blocks, and where the table segment of this wavefront's first group starts.
struct NearestList {
  int list;
  uint32_t len, nblk;
  int32_t dir;
};

template <int METRIC, int ST>
__device__ void sample_scores(const Dev &D, int nprobe, int max_nprobe, int q, uint32_t want_groups,
                              const float *__restrict__ Q, const SearchScratch &S, const float4 *qv,
                              uint32_t *skey, const NearestList &first) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int d4 = D.vchunks;  // 16-byte chunks of a stored vector
  constexpr int kPieces = pieces_of(ST);  // float4s of the query that go with a chunk
  const uint32_t gpb = (uint32_t)D.groups_per_block;
  const size_t group_stride = (size_t)d4 * kWave;
  // the sample is the first want_groups groups of the probed lists taken in order, nearest first
  uint32_t g_first = 0;  // groups of the lists before list p
  for (int p = 0; p < nprobe && g_first < want_groups; ++p) {  // uniform over the workgroup
    const size_t o = (size_t)q * max_nprobe + p;
    const int list = p == 0 ? first.list : S.probe_list[o];
    const uint32_t len = p == 0 ? first.len : S.probe_len[o];
    uint32_t groups = (len + kWave - 1) / kWave;
    const uint32_t have = (p == 0 ? first.nblk : D.nblk[list]) * gpb;  // never index the block table past the chain
    if (groups > have) groups = have;
    if (groups > want_groups - g_first) groups = want_groups - g_first;
    for (uint32_t g = (uint32_t)wave; g < groups; g += blockDim.x / kWave) {
      const uint32_t b = p == 0 && g == (uint32_t)wave ? (uint32_t)*table_entry_at(D, first.dir, g / gpb)
                                                       : (uint32_t)*table_entry(D, list, g / gpb);
      const float4 *__restrict__ x = block_vecs(D, b) + (size_t)(g % gpb) * group_stride + lane;
      float acc = 0.f;
      int c = 0;
      if (METRIC == 1 && ST == 0 && D.scan_mfma) {
        // inner products of float lists on the matrix cores, exactly as the scan computes them (same
        // instruction, same order of the coordinates), so that a candidate's score here and there is
        // the same bits: every lane offers the one query, component l % 4 of the result is the score
        // of the lane's own vector
        MfmaAcc m = {0.f, 0.f, 0.f, 0.f};
        for (; c + 8 <= d4; c += 8) {
          float4 v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) v[u] = x[(size_t)(c + u) * kWave];
#pragma unroll
          for (int u = 0; u < 8; ++u) mfma_chunk(m, v[u], qv[c + u]);
        }
        for (; c < d4; ++c) mfma_chunk(m, x[(size_t)c * kWave], qv[c]);
        const int r = lane & 3;
        acc = r == 0 ? m[0] : r == 1 ? m[1] : r == 2 ? m[2] : m[3];
      }
      // loads of 1 KiB in flight per wavefront: sixteen, then eight, then one at a time (the workgroup
      // is alone on its CU and a group is a chain of such round trips)
      if (ST == 0) {
        for (; c + 16 <= d4; c += 16) {
          float4 v[16];
#pragma unroll
          for (int u = 0; u < 16; ++u) v[u] = x[(size_t)(c + u) * kWave];
#pragma unroll
          for (int u = 0; u < 16; ++u) accumulate<METRIC>(acc, v[u], qv[c + u]);
        }
      }
      for (; c + 8 <= d4; c += 8) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = x[(size_t)(c + u) * kWave];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int s = 0; s < kPieces; ++s) accumulate<METRIC>(acc, chunk_piece<ST>(v[u], s), qv[(c + u) * kPieces + s]);
      }
      for (; c < d4; ++c) {
        const float4 v = x[(size_t)c * kWave];
#pragma unroll
        for (int s = 0; s < kPieces; ++s) accumulate<METRIC>(acc, chunk_piece<ST>(v, s), qv[c * kPieces + s]);
      }
      const uint32_t v = g * kWave + lane;
      skey[(size_t)(g_first + g) * kWave + lane] =
          v < len ? key_of_float((METRIC == 0 ? acc : -acc) + 0.0f) : 0xFFFFFFFFu;
    }
    g_first += groups;
  }
  // groups the lists did not have stay at the worst key (set by the caller)
}

// The same sample over product-quantiser codes: a vector's score is the sum, in the order of the
// sub-spaces, of the request's table entries that its codes name (the table stays in global
// memory here: a few thousand look-ups per query).
__device__ void pq_sample_scores(const Dev &D, int nprobe, int max_nprobe, int q, uint32_t want_groups,
                                 const SearchScratch &S, uint32_t *skey) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int words = D.pq_m / 4;
  const float *lut = S.lut + (size_t)q * D.pq_m * 256;
  const uint32_t gpb = (uint32_t)D.groups_per_block;
  uint32_t g_first = 0;
  for (int p = 0; p < nprobe && g_first < want_groups; ++p) {  // uniform over the workgroup
    const size_t o = (size_t)q * max_nprobe + p;
    const int list = S.probe_list[o];
    const uint32_t len = S.probe_len[o];
    uint32_t groups = (len + kWave - 1) / kWave;
    const uint32_t have = D.nblk[list] * gpb;  // never index the block table past the chain
    if (groups > have) groups = have;
    if (groups > want_groups - g_first) groups = want_groups - g_first;
    for (uint32_t g = (uint32_t)wave; g < groups; g += blockDim.x / kWave) {
      const uint32_t b = (uint32_t)*table_entry(D, list, g / gpb);
      const uint32_t *__restrict__ x = block_codes(D, b) + (size_t)(g % gpb) * words * kWave + lane;
      float acc = 0.f;
      for (int c = 0; c < words; ++c) {
        const uint32_t w = x[(size_t)c * kWave];
        const float *t = lut + (size_t)c * 4 * 256;
        acc += t[w & 255u];
        acc += t[256 + ((w >> 8) & 255u)];
        acc += t[512 + ((w >> 16) & 255u)];
        acc += t[768 + (w >> 24)];
      }
      const uint32_t v = g * kWave + lane;
      skey[(size_t)(g_first + g) * kWave + lane] =
          v < len ? key_of_float((D.metric == 0 ? acc : -acc) + 0.0f) : 0xFFFFFFFFu;
    }
    g_first += groups;
  }
}

// LDS of a bound: the query (d <= 2048) and the keys of the sample.  The caller owns it, so that a
// kernel whose workgroups do different jobs can use the same bytes for each.
constexpr size_t kBoundLdsBytes = 512 * sizeof(float4) + kSampleMax * sizeof(uint32_t);

template <bool PQ>
__device__ void sample_bound(const Dev &D, int q, int nprobe, int max_nprobe, int k, const float *__restrict__ Q,
                             const SearchScratch &S, unsigned char *lds) {
  float4 *qv = reinterpret_cast<float4 *>(lds);
  uint32_t *skey = reinterpret_cast<uint32_t *>(lds + 512 * sizeof(float4));
  __shared__ __attribute__((aligned(8))) uint32_t hist[kSelectLdsWords];
  __shared__ uint32_t bc[4];
  const int tid = threadIdx.x;
  // what decides how the workgroup goes on, all on its way at once
  const size_t o0 = (size_t)q * max_nprobe;
  const uint32_t qtotal = S.qtotal[q];
  NearestList first{PQ ? 0 : S.probe_list[o0], S.probe_len[o0], 0u, 0};
  // |q|^2 for the norm form of the squared distance (the first wavefront computes it, in double)
  const bool norm_form = !PQ && uses_norm_form(D);
  __shared__ float s_qn;
  if (norm_form && tid < kWave) {
    double a = 0.0;
    for (int c = tid; c < D.d; c += kWave) {
      const double v = (double)Q[(size_t)q * D.d + c];
      a = __builtin_fma(v, v, a);
    }
    for (int o = kWave / 2; o > 0; o >>= 1) a += __shfl_xor(a, o);
    if (tid == 0) { s_qn = (float)a; S.qnorm[q] = (float)a; }
  }
  // A query with no more candidates than the selection holds in LDS at once needs no bound.  For
  // inner products neither does one whose records cost less than a sample would: the sample is 512
  // vectors or more read by one workgroup (80 us at d = 768), a record is 8 bytes (short lists, wide
  // vectors).  (For L2 the bound also lets the scan stop early, which is worth the sample.)
  const uint32_t no_bound_below =
      D.metric == 0 ? (uint32_t)kNoBoundBelow : max((uint32_t)kNoBoundBelow, 32u * (uint32_t)D.d);
  if (qtotal <= no_bound_below) {  // uniform over the workgroup
    if (tid == 0) {
      S.bound[q] = 0xFFFFFFFFu;
      S.rec_cnt[q] = 0u;
    }
    return;
  }
  // sample size: 4 k, at least 512 and at least a fraction of the nearest list (the longer that
  // list, the more candidates a given score admits), at most kSampleMax and at most 1 MiB of
  // vectors (one workgroup reads the sample: a hot list of wide vectors would hold up the scan),
  // in whole groups
  uint32_t cap = PQ ? (uint32_t)kSampleMax : ((1u << 20) / ((uint32_t)D.vchunks * 16u)) & ~(uint32_t)(kWave - 1);
  cap = cap < 512u ? 512u : (cap > (uint32_t)kSampleMax ? (uint32_t)kSampleMax : cap);
  uint32_t want = (uint32_t)k * 4u;
  const uint32_t part = first.len / (uint32_t)kSampleDivisor;
  if (!PQ) {  // on their way while the query and the keys are set up
    first.nblk = D.nblk[first.list];
    first.dir = table_dir(D, first.list, (uint32_t)(tid / kWave) / (uint32_t)D.groups_per_block);
  }
  want = want < part ? part : want;
  want = want < 512u ? 512u : (want > cap ? cap : want);
  const uint32_t want_groups = (want + kWave - 1) / kWave;
  if (!PQ)
    for (int c = tid; c < D.d4; c += (int)blockDim.x) qv[c] = reinterpret_cast<const float4 *>(Q + (size_t)q * D.d)[c];
  for (int i = tid; i < (int)(want_groups * kWave); i += (int)blockDim.x) skey[i] = 0xFFFFFFFFu;
  __syncthreads();
  if (PQ) pq_sample_scores(D, nprobe, max_nprobe, q, want_groups, S, skey);
  else if (D.metric == 0) {
    if (D.storage == 1) sample_scores<0, 1>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey, first);
    else if (D.storage == 2) sample_scores<0, 2>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey, first);
    else sample_scores<0, 0>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey, first);
  } else {
    if (D.storage == 1) sample_scores<1, 1>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey, first);
    else if (D.storage == 2) sample_scores<1, 2>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey, first);
    else sample_scores<1, 0>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey, first);
  }
  __syncthreads();
  // k-th smallest key of the sample; with fewer than k candidates in it, it is the worst key
  // and everything is kept
  uint32_t bound = 0xFFFFFFFFu;
  if ((uint32_t)k <= want_groups * kWave) {
    const SelectResult r = wg_radix_select<32>(
        (int)(want_groups * kWave), (uint32_t)k, [&](int i, uint64_t &kv) { kv = skey[i]; return true; }, hist, bc);
    bound = (uint32_t)r.T;  // the k-th smallest key, or an upper bound of it that admits the same candidates
  }
  if (tid == 0) {
    // the sample's scores are direct-form ones; the scan may compare norm-form scores with the bound
    if (norm_form) bound = loosened_key(bound, norm_form_slack(D.d), s_qn);
    S.bound[q] = bound;
    S.rec_cnt[q] = 0u;
  }
}

// ------------------------------------------------------------ pair grouping
// The (query, probed list) pairs of a request are grouped by list, so that the
// scan reads a list once for up to tile_q queries (the scan kernel's choice).  One workgroup:
// prefix sums over the lists of the pair counts, the work-item counts and the
// work, then the item descriptors, the split of the items over the 8 XCDs and
// the grouped pair array.  A work item is (list, segment of seg_groups
// 64-vector groups, tile of up to tile_q of the queries probing the
// list); one wavefront walks it.  The items of one segment follow each other, so
// they run at the same time on the same CU or on its neighbours and the segment
// comes from HBM once.  Segments bound the work of one item, so that long lists
// spread over many wavefronts.  The segment length is the shortest power of two
// for which the request has at most `item_budget` items and no XCD more than
// `max_per_xcd` (the launch of the scan is sized from those two).
constexpr int kSegChoices = 8;  // segment lengths 2, 4, ..., 256 groups
constexpr int kLdsEntries = 1024;  // probed lists of a request up to which their entries stay in LDS
constexpr int kListChunk = 16;  // lists a thread of the grouping workgroup handles side by side

__device__ inline void wg_scan3(uint32_t &a, uint32_t &b, unsigned long long &c, uint32_t *sa,
                                uint32_t *sb, unsigned long long *sc) {
  // inclusive scan over the threads of three values at once: shuffles inside a
  // wavefront, then the wavefront totals through LDS; sa/sb/sc[kGroupThreads-1]
  // receive the grand totals
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  constexpr int kWaves = kGroupThreads / kWave;
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t xa = __shfl_up(a, o), xb = __shfl_up(b, o);
    const unsigned long long xc = __shfl_up(c, o);
    if (lane >= o) { a += xa; b += xb; c += xc; }
  }
  __syncthreads();  // earlier readers of the LDS arrays are done
  if (lane == kWave - 1) { sa[wave] = a; sb[wave] = b; sc[wave] = c; }
  __syncthreads();
  uint32_t oa = 0, ob = 0, ta = 0, tb = 0;
  unsigned long long oc = 0, tc = 0;
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t va = sa[w], vb = sb[w];
    const unsigned long long vc = sc[w];
    if (w < wave) { oa += va; ob += vb; oc += vc; }
    ta += va; tb += vb; tc += vc;
  }
  a += oa; b += ob; c += oc;
  __syncthreads();
  if (tid == kGroupThreads - 1) { sa[tid] = ta; sb[tid] = tb; sc[tid] = tc; }
  __syncthreads();
}

// The pairs of the request grouped by list: `grouped` holds, list after list in list order, the
// (query, probe) pairs that probe the list, each at the rank the plan gave it.  One workgroup, beside
// the one that cuts the work items (both derive the same pair starts from the same counters: a
// running sum of the pair counts over the lists, a row of consecutive lists per thread at a time, 16 rows in flight).
// Several workgroups may share the pairs (part `part` of `parts`): each derives all the starts (every
// one of them writes the same numbers to pair_start) and places its own share of the pairs.
__device__ void scatter_pairs(const Dev &D, int nq, int nprobe, int max_nprobe, const SearchScratch &S, int part,
                              int parts) {
  constexpr int kWavesG = kGroupThreads / kWave;
  __shared__ uint32_t s_tot[kListChunk * kWavesG + 1];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const uint32_t *__restrict__ list_cnt = S.list_cnt;
  uint32_t *__restrict__ pair_start = S.pair_start;
  uint32_t before = 0;  // pairs of the lists in front of the current rows
  for (int lb = 0; lb < D.nlist; lb += kListChunk * kGroupThreads) {  // uniform over the workgroup
    const int rows = min(kListChunk, (D.nlist - lb + kGroupThreads - 1) / kGroupThreads);
    uint32_t c[kListChunk], incl[kListChunk];
#pragma unroll
    for (int t = 0; t < kListChunk; ++t) {
      const int l = lb + t * kGroupThreads + tid;
      c[t] = t < rows && l < D.nlist ? list_cnt[l] : 0u;
    }
#pragma unroll
    for (int t = 0; t < kListChunk; ++t) {
      incl[t] = c[t];
      if (t < rows) {  // uniform
        for (int o = 1; o < kWave; o <<= 1) {
          const uint32_t x = __shfl_up(incl[t], o);
          if (lane >= o) incl[t] += x;
        }
        if (lane == kWave - 1) s_tot[t * kWavesG + wave] = incl[t];
      }
    }
    __syncthreads();
    if (wave == 0) {  // running sum over the (row, wavefront) totals, in list order
      uint32_t carry = 0;
      const int counts = rows * kWavesG;
      for (int i0 = 0; i0 < counts; i0 += kWave) {
        const uint32_t v = i0 + lane < counts ? s_tot[i0 + lane] : 0u;
        uint32_t in2 = v;
        for (int o = 1; o < kWave; o <<= 1) {
          const uint32_t x = __shfl_up(in2, o);
          if (lane >= o) in2 += x;
        }
        if (i0 + lane < counts) s_tot[i0 + lane] = carry + in2 - v;
        carry += __shfl(in2, kWave - 1);
      }
      if (lane == 0) s_tot[kListChunk * kWavesG] = carry;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < kListChunk; ++t)
      if (c[t]) pair_start[lb + t * kGroupThreads + tid] = before + s_tot[t * kWavesG + wave] + incl[t] - c[t];
    before += s_tot[kListChunk * kWavesG];
    __syncthreads();  // the totals are reused by the next rows; the starts are read below by other threads
  }
  // eight independent chains of loads per thread
  const int npairs_all = nq * nprobe;
  const int share = (npairs_all + parts - 1) / parts;
  const int npairs = min(npairs_all, (part + 1) * share);
  for (int base = part * share + tid; base < npairs; base += 8 * kGroupThreads) {
    int l[8];
    uint32_t slot[8], pk[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = base + u * kGroupThreads;
      if (idx < npairs) {
        const int q = idx / nprobe, p = idx - q * nprobe;
        const size_t o = (size_t)q * max_nprobe + p;
        l[u] = S.probe_list[o];
        slot[u] = S.pair_slot[o];
        pk[u] = ((uint32_t)q << 10) | (uint32_t)p;
      } else {
        l[u] = -1;
      }
    }
    uint32_t start[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) start[u] = l[u] >= 0 ? pair_start[l[u]] : 0u;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (l[u] >= 0) S.grouped[start[u] + slot[u]] = pk[u];
  }
}

// A thread's entries e0 .. e1 - 1, CH at a time: the loads of a chunk go out together, then body(e,
// entry) for every entry of the chunk that is probed.
template <int CH, typename Body>
__device__ __forceinline__ void walk_entries(const uint4 *plist, uint32_t e0, uint32_t e1, Body body) {
  for (uint32_t eb = e0; eb < e1; eb += CH) {
    uint4 pl[CH];
#pragma unroll
    for (int t = 0; t < CH; ++t) pl[t] = eb + t < e1 ? plist[eb + t] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int t = 0; t < CH; ++t)
      if (pl[t].z) body(eb + (uint32_t)t, pl[t]);
  }
}

__global__ __launch_bounds__(kGroupThreads, 4) void k_group(Dev D, int nq, int nprobe, int max_nprobe, int k,
                                                         const float *__restrict__ Q,
                                                         uint32_t item_budget, uint32_t max_per_xcd,
                                                         uint32_t tile_q, int min_choice, int scatterers,
                                                         SearchScratch S) {
  const int tile_shift = 31 - __clz((int)tile_q);  // tiles hold a power of two of queries
  if (blockIdx.x >= 1 && (int)blockIdx.x <= scatterers) {  // uniform over the workgroup: these group the pairs by list
    scatter_pairs(D, nq, nprobe, max_nprobe, S, (int)blockIdx.x - 1, scatterers);
    return;
  }
  // the bound's query and sample keys, or the entries of the probed lists of a small request
  __shared__ __attribute__((aligned(16))) unsigned char s_raw[kBoundLdsBytes];
  static_assert(kBoundLdsBytes >= kLdsEntries * (sizeof(uint4) + sizeof(uint32_t)), "the entries share the bound's LDS");
  if (blockIdx.x > 0) {  // this one sets the bound of a query
    sample_bound<false>(D, (int)blockIdx.x - 1 - scatterers, nprobe, max_nprobe, k, Q, S, s_raw);
    return;
  }
  __shared__ uint32_t s_a[kGroupThreads];
  __shared__ uint32_t s_b[kGroupThreads];
  __shared__ unsigned long long s_c[kGroupThreads];
  __shared__ uint32_t s_items[kSegChoices];
  __shared__ uint32_t s_begin[9];
  constexpr uint32_t kHugeItems = 512, kHugeCap = 64;  // lists with this many items: at most so many are spread over the workgroup
  __shared__ uint4 s_huge_pl[kHugeCap];
  __shared__ uint32_t s_huge_ist[kHugeCap];
  __shared__ uint32_t s_nhuge;
  __shared__ uint32_t s_rows[kListChunk * (kGroupThreads / kWave) + 1];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  if (tid == 0) s_nhuge = 0;
  const uint32_t *__restrict__ list_cnt = S.list_cnt;
  uint4 *__restrict__ tile_desc = S.tile_desc;
  // The entries of the probed lists are written by one thread and read by another several times
  // over: every such hand-over through global memory is a round trip of a microsecond that nothing
  // hides (this workgroup is alone on its CU).  A request that can probe at most kLdsEntries
  // different lists keeps them in LDS.
  const bool lean = (long long)min((long long)D.nlist, (long long)nq * nprobe) <= kLdsEntries;
  uint4 *plist = lean ? reinterpret_cast<uint4 *>(s_raw) : S.plist;
  uint32_t *pistart = lean ? reinterpret_cast<uint32_t *>(s_raw + kLdsEntries * sizeof(uint4)) : S.pistart;
  ScanQueues *Qs = S.queues;
  // Cost of a list for the split over the XCDs, per group of 64 vectors: reading it once from HBM
  // (each XCD has its own link to memory) plus the arithmetic of every query that probes it.  On
  // this chip one group's bytes cost about as much as the arithmetic of 12 queries (L2) or 24 (IP).
  const uint32_t byte_weight = D.scan_byte_weight > 0 ? (uint32_t)D.scan_byte_weight : D.metric == 0 ? 12u : 24u;

  // The probed lists, compacted in list order (neighbouring lists sit in neighbouring blocks after a
  // bulk load, and the scan reads faster in that order): entry = {list, first pair, pairs, length}.
  // The pair counters are read a row of consecutive lists (one per thread) at a time, 16 such rows in flight;
  // the place of a probed list among the entries comes from ballots and one small prefix sum.  Lists
  // nobody probes are not looked at again (16,384 lists, 256 x 64 pairs: a quarter of the lists).
  // The visible length of every probed list is read ONCE: an insertion may publish while this kernel
  // runs, and the passes below must agree on the segment counts.  (Each pair's own snapshot was
  // taken earlier, so it is not longer than this one.)
  uint32_t n_c = 0;
  uint32_t cnt[kSegChoices];  // work items of this thread's lists for every segment length
#pragma unroll
  for (int e = 0; e < kSegChoices; ++e) cnt[e] = 0;
  if (tid < kSegChoices) s_items[tid] = 0;
  constexpr int kWavesG = kGroupThreads / kWave;
  for (int lb = 0; lb < D.nlist; lb += kListChunk * kGroupThreads) {  // uniform over the workgroup
    const int rows = min(kListChunk, (D.nlist - lb + kGroupThreads - 1) / kGroupThreads);
    uint32_t c[kListChunk];
    unsigned long long flags[kListChunk];
#pragma unroll
    for (int t = 0; t < kListChunk; ++t) {
      const int l = lb + t * kGroupThreads + tid;
      c[t] = t < rows && l < D.nlist ? list_cnt[l] : 0u;
    }
#pragma unroll
    for (int t = 0; t < kListChunk; ++t) {
      flags[t] = 0ull;
      if (t < rows) {  // uniform
        flags[t] = __ballot(c[t] != 0u);
        if (lane == 0) s_rows[t * kWavesG + wave] = (uint32_t)__popcll(flags[t]);
      }
    }
    __syncthreads();
    if (wave == 0) {  // running sum over the (row, wavefront) counts, in list order
      uint32_t carry = 0;
      const int counts = rows * kWavesG;
      for (int i0 = 0; i0 < counts; i0 += kWave) {
        const uint32_t v = i0 + lane < counts ? s_rows[i0 + lane] : 0u;
        uint32_t incl = v;
        for (int o = 1; o < kWave; o <<= 1) {
          const uint32_t x = __shfl_up(incl, o);
          if (lane >= o) incl += x;
        }
        if (i0 + lane < counts) s_rows[i0 + lane] = carry + incl - v;
        carry += __shfl(incl, kWave - 1);
      }
      if (lane == 0) s_rows[kListChunk * kWavesG] = carry;
    }
    __syncthreads();
    uint32_t len[kListChunk];
#pragma unroll
    for (int t = 0; t < kListChunk; ++t)
      len[t] = c[t] ? __hip_atomic_load(&D.visible_len[lb + t * kGroupThreads + tid], __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_AGENT)
                    : 0u;
#pragma unroll
    for (int t = 0; t < kListChunk; ++t) {
      if (!c[t]) continue;
      const uint32_t at =
          n_c + s_rows[t * kWavesG + wave] + (uint32_t)__popcll(flags[t] & ((1ull << lane) - 1ull));
      plist[at] = make_uint4((uint32_t)(lb + t * kGroupThreads + tid), 0u, c[t], len[t]);
      const uint32_t groups = (len[t] + kWave - 1) / kWave;
      const uint32_t tiles = (c[t] + tile_q - 1) >> tile_shift;
#pragma unroll
      for (int e = 0; e < kSegChoices; ++e) {
        const uint32_t sg = 2u << e;
        cnt[e] += (groups ? (groups + sg - 1) / sg : 1u) * tiles;
      }
    }
    n_c += s_rows[kListChunk * kWavesG];
    __syncthreads();  // the counts are reused by the next rows; the entries are read below by other threads
  }
  // totals per segment length: shuffles inside the wavefront, one LDS atomic per wavefront
  // (every lane adding to the same LDS word would serialise)
#pragma unroll
  for (int e = 0; e < kSegChoices; ++e) {
    uint32_t v = cnt[e];
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if (lane == 0 && v) atomicAdd(&s_items[e], v);
  }
  // From here on a thread owns `per` consecutive entries and walks them kListChunk at a time, so
  // that the loads of a chunk go out together: a pass over the entries is a chain of memory
  // latencies otherwise.  (With one or two entries to a thread the chunk is two wide: sixteen
  // guarded loads, each waited for by itself, cost a small request three microseconds a pass.)
  const uint32_t per = (n_c + kGroupThreads - 1) / kGroupThreads;
  const uint32_t e0 = min(n_c, (uint32_t)tid * per), e1 = min(n_c, e0 + per);
  auto for_my_entries = [&](auto body) {
    if (per <= 2) walk_entries<2>(plist, e0, e1, body);  // uniform over the workgroup
    else walk_entries<kListChunk>(plist, e0, e1, body);
  };
  __syncthreads();
  int choice = kSegChoices - 1;
  for (int e = min_choice; e < kSegChoices; ++e)
    if (s_items[e] <= item_budget && s_items[e] <= S.item_cap) { choice = e; break; }

  for (;; ++choice) {  // uniform: every thread sees the same totals
    const uint32_t seg = 2u << choice;
    uint32_t np = 0, ni = 0;
    unsigned long long wk = 0;
    for_my_entries([&](uint32_t, const uint4 &pl) {
      const uint32_t c = pl.z;
      const uint32_t groups = (pl.w + kWave - 1) / kWave;
      np += c;
      ni += (groups ? (groups + seg - 1) / seg : 1u) * ((c + tile_q - 1) >> tile_shift);
      wk += (unsigned long long)(c + byte_weight) * (groups ? groups : 1u);
    });
    uint32_t inp = np, ini = ni;
    unsigned long long iwk = wk;
    wg_scan3(inp, ini, iwk, s_a, s_b, s_c);
    const uint32_t total_items = s_b[kGroupThreads - 1];
    const unsigned long long total_work = s_c[kGroupThreads - 1];
    const uint32_t pstart0 = inp - np, istart0 = ini - ni;
    const unsigned long long wstart0 = iwk - wk;
    // XCD x starts at the item at which the work prefix passes x/8 of the total
    if (tid < 9) s_begin[tid] = tid == 8 ? total_items : 0u;
    __syncthreads();
    {
      uint32_t is = istart0;
      unsigned long long ws = wstart0;
      for_my_entries([&](uint32_t, const uint4 &pl) {
        const uint32_t c = pl.z;
        const uint32_t groups = (pl.w + kWave - 1) / kWave;
        const unsigned long long w = (unsigned long long)(c + byte_weight) * (groups ? groups : 1u);
        const uint32_t n = (groups ? (groups + seg - 1) / seg : 1u) * ((c + tile_q - 1) >> tile_shift);
        for (uint32_t x = 1; x < 8; ++x) {  // the cut falls inside this list: at the item the same share of it ends at
          const unsigned long long cut = total_work * x / 8;
          if (ws <= cut && cut < ws + w) s_begin[x] = is + (uint32_t)((cut - ws) * n / w);
        }
        is += n;
        ws += w;
      });
    }
    __syncthreads();
    if (tid == 0)  // several cuts may fall into one list: keep the sequence monotone
      for (uint32_t x = 1; x < 8; ++x)
        if (s_begin[x] < s_begin[x - 1]) s_begin[x] = s_begin[x - 1];
    __syncthreads();
    uint32_t longest = 0;
    for (uint32_t x = 0; x < 8; ++x) longest = max(longest, s_begin[x + 1] - s_begin[x]);
    if (longest > max_per_xcd) {  // uniform.  Items of very unequal cost: give every XCD the same number instead
      __syncthreads();
      if (tid < 9) s_begin[tid] = (uint32_t)((unsigned long long)total_items * tid / 8);
      __syncthreads();
      longest = (total_items + 7) / 8;
    }
    const bool fits = total_items <= S.item_cap && longest <= max_per_xcd;
    if (!fits && choice + 1 < kSegChoices + 8) continue;  // coarser segments (bounded: lengths are 32 bit)
    if (tid < 9) Qs->begin[tid] = s_begin[tid];
    if (tid == 0) {
      Qs->seg_groups = fits ? seg : 0u;
      if (!fits) {  // more tiles than the request's item descriptors hold: nothing is scanned, and the caller is told
        atomicCAS(&D.ctrl->search_error, 0, -6);
        D.mirror->search_error = -6;
      }
    }
    // where the pairs and the items of every probed list start
    {
      uint32_t ps = pstart0, is = istart0;
      for_my_entries([&](uint32_t e, const uint4 &pl) {
        const uint32_t c = pl.z;
        const uint32_t groups = (pl.w + kWave - 1) / kWave;
        plist[e] = make_uint4(pl.x, ps, c, pl.w);
        pistart[e] = is;
        ps += c;
        is += (groups ? (groups + seg - 1) / seg : 1u) * ((c + tile_q - 1) >> tile_shift);
      });
    }
    __syncthreads();  // entries written above are read below by other threads
    // Item descriptors.  A wavefront takes a sixteenth of the entries, 64 at a time, lane = entry.
    // Most lists have a handful of items: their lane writes them itself.  A list with more is taken
    // by the whole wavefront, the lanes writing its items side by side, and one with very many (a
    // hot list probed by dozens of queries has thousands) by the whole workgroup afterwards.  Inside a list the tiles of one segment follow each other,
    // and the tiles are of (almost) equal size.
    if (fits) {
      constexpr uint32_t kWaves = kGroupThreads / kWave;
      constexpr uint32_t kOwnItems = 16;
      const uint32_t w0 = (uint32_t)((unsigned long long)n_c * wave / kWaves);
      const uint32_t w1 = (uint32_t)((unsigned long long)n_c * (wave + 1) / kWaves);
      for (uint32_t eb = w0; eb < w1; eb += kWave) {
        const uint32_t mine = eb + (uint32_t)lane;
        const uint4 pl = mine < w1 ? plist[mine] : make_uint4(0u, 0u, 0u, 0u);
        const uint32_t ist = mine < w1 ? pistart[mine] : 0u;
        uint32_t n = 0, tiles = 1, small = 0, extra = 0;
        if (pl.z) {
          const uint32_t groups = (pl.w + kWave - 1) / kWave;
          tiles = (pl.z + tile_q - 1) >> tile_shift;
          n = (groups ? (groups + seg - 1) / seg : 1u) * tiles;
          small = pl.z / tiles;
          extra = pl.z - small * tiles;  // the first `extra` tiles hold one more
        }
        if (n <= kOwnItems) {
          uint32_t sg = 0, tt = 0;
          for (uint32_t i = 0; i < n; ++i) {
            const uint32_t p_lo = tt * small + min(tt, extra);
            tile_desc[ist + i] = make_uint4(pl.x, pl.y + p_lo, small + (tt < extra ? 1u : 0u), sg);
            if (++tt == tiles) { tt = 0; ++sg; }
          }
        }
        // the few lists with very many items are left to the whole workgroup (below)
        bool huge = n >= kHugeItems;
        if (huge) {
          const uint32_t slot = atomicAdd(&s_nhuge, 1u);
          if (slot < kHugeCap) {
            s_huge_pl[slot] = pl;
            s_huge_ist[slot] = ist;
          } else {
            huge = false;  // no room: the wavefront takes it after all
          }
        }
        unsigned long long big = __ballot(n > kOwnItems && !huge);
        while (big) {  // uniform over the wavefront
          const int t = __builtin_ctzll(big);
          big &= big - 1;
          const uint32_t l = (uint32_t)__shfl((int)pl.x, t), ps = (uint32_t)__shfl((int)pl.y, t);
          const uint32_t first = (uint32_t)__shfl((int)ist, t), n_t = (uint32_t)__shfl((int)n, t);
          const uint32_t tiles_t = (uint32_t)__shfl((int)tiles, t);
          const uint32_t small_t = (uint32_t)__shfl((int)small, t), extra_t = (uint32_t)__shfl((int)extra, t);
          for (uint32_t i = (uint32_t)lane; i < n_t; i += kWave) {
            const uint32_t sg = i / tiles_t, tt = i - sg * tiles_t;
            const uint32_t p_lo = tt * small_t + min(tt, extra_t);
            tile_desc[first + i] = make_uint4(l, ps + p_lo, small_t + (tt < extra_t ? 1u : 0u), sg);
          }
        }
      }
    }
    __syncthreads();
    if (fits) {
      const uint32_t nh = min(s_nhuge, kHugeCap);
      for (uint32_t h = 0; h < nh; ++h) {  // uniform over the workgroup
        const uint4 pl = s_huge_pl[h];
        const uint32_t first = s_huge_ist[h];
        const uint32_t groups = (pl.w + kWave - 1) / kWave;
        const uint32_t tiles = (pl.z + tile_q - 1) >> tile_shift;
        const uint32_t n = (groups ? (groups + seg - 1) / seg : 1u) * tiles;
        const uint32_t small = pl.z / tiles, extra = pl.z - small * tiles;
        for (uint32_t i = (uint32_t)tid; i < n; i += kGroupThreads) {
          const uint32_t sg = i / tiles, tt = i - sg * tiles;
          const uint32_t p_lo = tt * small + min(tt, extra);
          tile_desc[first + i] = make_uint4(pl.x, pl.y + p_lo, small + (tt < extra ? 1u : 0u), sg);
        }
      }
    }
    break;
  }
}


constexpr int kPqBoundThreads = 1024;

// The bound of every query of a request over quantised lists (the grouping by list that the scan
// of flat lists needs is not made).
// The workgroup of a query first writes the query's table of sub-scores: lut[q][m][c] = squared
// distance (L2) or inner product (IP) between sub-vector m of the query and entry c of codebook m,
// fp32, one FMA chain in the order of the dimensions; its sample and the scan read it from there.
__global__ __launch_bounds__(kPqBoundThreads) void k_pq_bound(Dev D, int nprobe, int max_nprobe, int k,
                                                            const float *__restrict__ Q, SearchScratch S) {
  const int q = blockIdx.x;
  {
    const int M = D.pq_m, ds = D.d / M;
    const float *__restrict__ yq = Q + (size_t)q * D.d;
    float *__restrict__ lut = S.lut + (size_t)q * M * 256;
    // M * 256 entries, 1024 threads: M / 4 rounds, four of them side by side (their loads overlap);
    // 16-byte loads where the sub-space allows
    for (int i0 = threadIdx.x; i0 < M * 256; i0 += 4 * kPqBoundThreads) {
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      if (ds % 4 == 0) {  // uniform
        for (int j4 = 0; j4 < ds / 4; ++j4) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int i = i0 + r * kPqBoundThreads;
            if (i < M * 256) {
              const float4 ev = reinterpret_cast<const float4 *>(D.codebooks + (size_t)i * ds)[j4];
              const float4 yv = reinterpret_cast<const float4 *>(yq + (size_t)(i >> 8) * ds)[j4];
              if (D.metric == 0) {
                const float u0 = ev.x - yv.x, u1 = ev.y - yv.y, u2 = ev.z - yv.z, u3 = ev.w - yv.w;
                acc[r] = fmaf(u0, u0, acc[r]); acc[r] = fmaf(u1, u1, acc[r]);
                acc[r] = fmaf(u2, u2, acc[r]); acc[r] = fmaf(u3, u3, acc[r]);
              } else {
                acc[r] = fmaf(ev.x, yv.x, acc[r]); acc[r] = fmaf(ev.y, yv.y, acc[r]);
                acc[r] = fmaf(ev.z, yv.z, acc[r]); acc[r] = fmaf(ev.w, yv.w, acc[r]);
              }
            }
          }
        }
      } else {
        for (int j = 0; j < ds; ++j) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int i = i0 + r * kPqBoundThreads;
            if (i < M * 256) {
              const float ev = D.codebooks[(size_t)i * ds + j], yv = yq[(size_t)(i >> 8) * ds + j];
              if (D.metric == 0) { const float u = ev - yv; acc[r] = fmaf(u, u, acc[r]); }
              else acc[r] = fmaf(ev, yv, acc[r]);
            }
          }
        }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (i0 + r * kPqBoundThreads < M * 256) lut[i0 + r * kPqBoundThreads] = acc[r];
    }
  }
  __threadfence_block();
  __syncthreads();  // the sample below reads the table
  __shared__ __attribute__((aligned(16))) unsigned char s_raw[kBoundLdsBytes];
  sample_bound<true>(D, q, nprobe, max_nprobe, k, nullptr, S, s_raw);
}


void launch_group(const Dev &D, int64_t nq, int nprobe, int max_nprobe, int k, const float *Q,
                  int item_budget, const SearchScratch &S, hipStream_t s) {
  if (nq <= 0) return;
  if (D.pq_m > 0) {
    hipLaunchKernelGGL(k_pq_bound, dim3((unsigned)nq), dim3(kPqBoundThreads), 0, s, D, nprobe, max_nprobe, k, Q, S);
    return;
  }
  // workgroup 0 cuts the work items, the next few group the pairs (one for every 2048 pairs, at most 8:
  // placing a pair is a chain of three round trips to memory), the others set the bound of a query each
  const ScanShape sh = scan_shape(D, item_budget);
  const int64_t pairs = nq * nprobe;
  const int scatterers = (int)(pairs <= 2048 ? 1 : pairs >= 8 * 2048 ? 8 : (pairs + 2047) / 2048);
  hipLaunchKernelGGL(k_group, dim3(1 + (unsigned)scatterers + (unsigned)nq), dim3(kGroupThreads), 0, s, D, (int)nq,
                     nprobe, max_nprobe, k, Q, (uint32_t)item_budget,
                     (uint32_t)(sh.grid / (int)kXcds * sh.items_per_wg), (uint32_t)sh.tile_q, sh.min_choice,
                     scatterers, S);
}

}  // namespace rtams
