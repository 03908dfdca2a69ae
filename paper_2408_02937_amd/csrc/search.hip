// Search path: probe selection and plan, list scan, top-k selection.
// (Paper, introduction: a query is compared with the lists of the clusters nearest to it only, and
// the k best of those come back; distances are exact, so the result is the textbook IVF-Flat one.)
#include "rtams_launch.h"

namespace rtams {

constexpr int kSelThreads = 256;

// ------------------------------------------------------------------ key maps
// Monotone maps from scores to unsigned keys: a smaller key is a better score.
__device__ inline uint64_t key_of_double(double x) {
  uint64_t b = (uint64_t)__double_as_longlong(x);
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ inline uint32_t key_of_float(float x) {
  uint32_t b = __float_as_uint(x);
  return (b >> 31) ? ~b : (b | 0x80000000u);
}

// ------------------------------------------------------- survivor records
// Where a query's records lie: in its request's slice or, flagged, in the reserve all resources share.
__device__ inline uint32_t *rec_keys_of(const SearchScratch &S, unsigned long long qbase) {
  return (qbase & kInOverflow) ? S.ovf_key + (qbase & ~kInOverflow) : S.rec_key + qbase;
}
__device__ inline uint32_t *rec_poss_of(const SearchScratch &S, unsigned long long qbase) {
  return (qbase & kInOverflow) ? S.ovf_pos + (qbase & ~kInOverflow) : S.rec_pos + qbase;
}
// Room for `want` entries in the request's chunk of the shared reserve (called by one thread per
// query): the start, flagged, or ~0.  The first query of a request that needs it leases a free chunk
// and installs it for the request; one that loses that race to a sibling hands its chunk straight
// back and shares the sibling's.  Nothing here waits for anybody.
__device__ inline unsigned long long overflow_take(const SearchScratch &S, unsigned long long want) {
  if (S.ovf_chunks == 0 || want > S.ovf_chunk_cap) return ~0ull;
  uint32_t c = __hip_atomic_load(S.req_chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (uint32_t e = 0; e < S.ovf_chunks && c == 0; ++e)
    if (atomicCAS(&S.ovf_leased[e], 0u, 1u) == 0u) {
      const uint32_t seen = atomicCAS(S.req_chunk, 0u, e + 1u);
      if (seen == 0u) c = e + 1u;
      else { atomicExch(&S.ovf_leased[e], 0u); c = seen; }
    }
  if (c == 0) c = __hip_atomic_load(S.req_chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // a sibling may have got the last one
  if (c == 0) return ~0ull;  // every chunk is out
  const unsigned long long off = atomicAdd(S.req_cursor, want);
  if (off + want > S.ovf_chunk_cap) return ~0ull;
  return kInOverflow | ((unsigned long long)(c - 1u) * S.ovf_chunk_cap + off);
}
// Every selection workgroup of a request reports here when it has read its last record; the last
// one returns the request's chunk, if it holds one, and resets the request's words.
__device__ inline void overflow_request_done(const SearchScratch &S, uint32_t workgroups) {
  if (S.ovf_chunks == 0) return;
  __threadfence();
  if (atomicAdd(S.req_done, 1u) + 1u != workgroups) return;
  const uint32_t c = __hip_atomic_load(S.req_chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(S.req_done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(S.req_cursor, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (c) {
    __hip_atomic_store(S.req_chunk, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();
    atomicExch(&S.ovf_leased[c - 1u], 0u);
  }
}

// ------------------------------------------------- workgroup radix selection
// Finds the threshold of the k smallest keys among the valid items 0..n-1.
// fn(i, key) returns false for items that do not take part.  On return T is
// a threshold such that every key < T belongs to the k smallest and, of the
// c_eq keys not yet told apart from T, `need` belong to them (when c_eq == need
// the selection stops early and T is the largest key that group can hold; else
// T is the k-th smallest key itself and the c_eq keys equal it).  Callers take
// key < T, and key == T under the tie rule.  Requires 1 <= k <= #valid.
struct SelectResult {
  uint64_t T;
  uint32_t need, c_eq;
};

// After a histogram pass: the first wavefront finds the bin that holds the
// need-th smallest item; bc = {bin, items in lower bins, items in the bin}.
__device__ inline void wg_pick_bin(const uint32_t *hist, uint32_t need, uint32_t *bc) {
  if (threadIdx.x < kWave) {  // first wavefront: which bin holds the need-th item
      int l = threadIdx.x;
      uint32_t h0 = hist[4 * l], h1 = hist[4 * l + 1], h2 = hist[4 * l + 2], h3 = hist[4 * l + 3];
      uint32_t sum = h0 + h1 + h2 + h3, incl = sum;
      for (int o = 1; o < kWave; o <<= 1) {
        uint32_t t = __shfl_up(incl, o);
        if (l >= o) incl += t;
      }
      uint32_t excl = incl - sum;
      if (excl < need && need <= incl) {  // exactly one lane
        uint32_t cum = excl;
        int dg;
        uint32_t hh;
        if (cum + h0 >= need) { dg = 0; hh = h0; }
        else { cum += h0;
          if (cum + h1 >= need) { dg = 1; hh = h1; }
          else { cum += h1;
            if (cum + h2 >= need) { dg = 2; hh = h2; }
            else { cum += h2; dg = 3; hh = h3; } } }
        bc[0] = (uint32_t)(4 * l + dg);
        bc[1] = cum;
        bc[2] = hh;
      }
    }
    __syncthreads();
}

// `each(body)` calls body(key) for every key of the calling thread that takes part.
template <int BITS, typename Each>
__device__ SelectResult wg_radix_select_each(uint32_t k, Each each, uint32_t *hist, uint32_t *bc) {
  // Leading digits on which every key agrees are skipped: scores of one query's
  // candidates share sign, exponent and often the first mantissa bits, and a
  // histogram pass in which all lanes hit one LDS word serialises completely.
  unsigned long long *mm = reinterpret_cast<unsigned long long *>(hist);  // {min, max} for a moment
  if (threadIdx.x == 0) { mm[0] = ~0ull; mm[1] = 0ull; }
  __syncthreads();
  {
    unsigned long long lo = ~0ull, hi = 0ull;
    each([&](uint64_t key) { lo = key < lo ? key : lo; hi = key > hi ? key : hi; });
    for (int o = kWave / 2; o > 0; o >>= 1) {
      const unsigned long long a = __shfl_xor(lo, o), b = __shfl_xor(hi, o);
      lo = a < lo ? a : lo;
      hi = b > hi ? b : hi;
    }
    if ((threadIdx.x & (kWave - 1)) == 0) { atomicMin(&mm[0], lo); atomicMax(&mm[1], hi); }
  }
  __syncthreads();
  const uint64_t kmin = mm[0], kmax = mm[1];
  __syncthreads();  // hist is reused below
  int first_shift = BITS - 8;
  uint64_t prefix = 0, mask = 0;
  {
    const uint64_t diff = kmin ^ kmax;
    const int top = diff ? 63 - __clzll((long long)diff) : -1;  // highest bit in which keys differ
    first_shift = top < 0 ? 0 : (top / 8) * 8;
    if (first_shift > BITS - 8) first_shift = BITS - 8;
    if (first_shift + 8 < 64) {
      mask = ~0ull << (first_shift + 8);
      if (BITS < 64) mask &= (1ull << BITS) - 1ull;
    }
    prefix = kmax & mask;
  }
  uint32_t need = k, c_eq = 0;
  for (int shift = first_shift; shift >= 0; shift -= 8) {
    for (int b = threadIdx.x; b < 256; b += blockDim.x) hist[b] = 0;
    __syncthreads();
    each([&](uint64_t key) {
      if ((key & mask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & 255u], 1u);
    });
    __syncthreads();
    wg_pick_bin(hist, need, bc);
    uint32_t dg = bc[0];
    need -= bc[1];
    c_eq = bc[2];
    prefix |= (uint64_t)dg << shift;
    mask |= (uint64_t)255u << shift;
    __syncthreads();
    if (c_eq == need) {  // the whole bin belongs to the k smallest: the lower digits cannot matter
      if (shift > 0) prefix |= (1ull << shift) - 1ull;  // threshold = largest key of the bin
      break;
    }
  }
  return {prefix, need, c_eq};
}

// Items 0..n-1 given by fn(i, key) (false: the item does not take part); keys are
// read from memory, four independent loads in flight per thread.
template <int BITS, typename Fn>
__device__ SelectResult wg_radix_select(int n, uint32_t k, Fn fn, uint32_t *hist, uint32_t *bc) {
  auto each = [&](auto body) {
    for (int i0 = threadIdx.x; i0 < n; i0 += 4 * blockDim.x) {
      uint64_t key[4];
      bool ok[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {  // clamped index: the loads are unconditional and issue back to back
        const int i = i0 + u * (int)blockDim.x;
        ok[u] = fn(i < n ? i : n - 1, key[u]) && i < n;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (ok[u]) body(key[u]);
    }
  };
  return wg_radix_select_each<BITS>(k, each, hist, bc);
}

// Bitonic sort of m (power of two) entries in LDS by (k1, k2) ascending; pay is
// carried along.  The first wavefront does all of it (LDS operations of one
// wavefront execute in order, so the steps need no workgroup barrier); the
// others wait at the end.
__device__ inline void wg_bitonic_sort(int m, uint64_t *k1, uint64_t *k2, uint32_t *pay) {
  __syncthreads();
  if (threadIdx.x < kWave) {
    for (int size = 2; size <= m; size <<= 1) {
      for (int stride = size >> 1; stride > 0; stride >>= 1) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (int t = threadIdx.x; t < m / 2; t += kWave) {
          int i = 2 * t - (t & (stride - 1));
          int j = i + stride;
          bool up = (i & size) == 0;
          uint64_t a1 = k1[i], a2 = k2[i], b1 = k1[j], b2 = k2[j];
          bool a_gt_b = a1 != b1 ? a1 > b1 : a2 > b2;
          if (a_gt_b == up) {
            k1[i] = b1; k2[i] = b2; k1[j] = a1; k2[j] = a2;
            uint32_t p = pay[i]; pay[i] = pay[j]; pay[j] = p;
          }
        }
      }
    }
  }
  __syncthreads();
}

__device__ inline int next_pow2(int v) {
  int m = 1;
  while (m < v) m <<= 1;
  return m;
}

// Sort of the first n entries in LDS by (k1, k2) ascending, pay carried along; entries from n up to
// the next power of two may be overwritten.  A few hundred entries at most are ranked: a group
// of S neighbouring lanes counts, each over its share of the entries, how many come before entry
// e (equal pairs in the order they stand in), and the entry is written to that place — two
// barriers instead of the dozens of dependent LDS round trips of a sorting network, which costs a
// single wavefront 5 to 7 us for 32 to 128 entries.  More entries go through the network.
constexpr int kRankSortMax = 256;
__device__ inline void wg_sort(int n, uint64_t *k1, uint64_t *k2, uint32_t *pay) {
  const int T = (int)blockDim.x;
  if (n > kRankSortMax || n > T) {  // uniform over the workgroup
    const int m = next_pow2(n > 0 ? n : 1);
    __syncthreads();
    for (int p = n + (int)threadIdx.x; p < m; p += T) { k1[p] = ~0ull; k2[p] = ~0ull; pay[p] = 0; }
    wg_bitonic_sort(m, k1, k2, pay);
    return;
  }
  __syncthreads();
  int S = 1;  // lanes per entry: a power of two, at most a wavefront, S * n <= T
  while (S < kWave && 2 * S * n <= T) S *= 2;
  const int e = (int)threadIdx.x / S, s = (int)threadIdx.x % S;
  const bool on = e < n;
  uint64_t a1 = 0, a2 = 0;
  uint32_t ap = 0, before = 0;
  if (on) {
    a1 = k1[e]; a2 = k2[e]; ap = pay[e];
    const int per = (n + S - 1) / S;
    const int lo = s * per, hi = lo + per < n ? lo + per : n;
    for (int j = lo; j < hi; ++j) {
      const uint64_t b1 = k1[j], b2 = k2[j];
      before += (b1 < a1 || (b1 == a1 && (b2 < a2 || (b2 == a2 && j < e)))) ? 1u : 0u;
    }
  }
  for (int o = 1; o < S; o <<= 1) before += __shfl_xor(before, o);  // the S lanes of an entry are neighbours in one wavefront
  __syncthreads();  // everybody has read
  if (on && s == 0) { k1[before] = a1; k2[before] = a2; pay[before] = ap; }
  __syncthreads();
}

// ------------------------------------------------------------ probe and plan
// One workgroup per query: the nprobe best centroids by (score, index), best
// first; then the plan of the scan: the visible length of each probed list is
// read ONCE here, so that scan and selection agree on it whatever an insertion
// publishes meanwhile, and the query gets its slice of the candidate array.
// FROM_APPROX: the request's coarse scores are fp32 approximations from the
// matrix cores (coarse_mfma.hip).  The nprobe-th smallest of them plus the error
// band bounds every centroid that can be among the exact nprobe best; those
// candidates are scored in the fixed double arithmetic here and ordered
// exactly.  If the band holds more candidates than LDS, the whole row is scored
// exactly instead (what small requests, which skip the matrix cores, always do).
template <bool FROM_APPROX>
__global__ __launch_bounds__(kSelThreads) void k_probe_plan(Dev D, int nprobe, int max_nprobe,
                                                            SearchScratch S, const float *__restrict__ Q,
                                                            int32_t *probe_out) {
  __shared__ __attribute__((aligned(8))) uint32_t hist[256];  // also holds two 64-bit words for a moment
  __shared__ uint32_t bc[4];
  __shared__ uint32_t cnt[2];
  __shared__ uint64_t k1[kMaxNprobe];
  __shared__ uint64_t k2[kMaxNprobe];
  __shared__ uint32_t pay[kMaxNprobe];
  __shared__ float s_red[kSelThreads / kWave];
  const int q = blockIdx.x;
  const int n = D.nlist;
  double *sc = S.scores + (size_t)q * n;
  const int metric = D.metric;
  auto exact = [&](int c) -> double {  // the fixed arithmetic of coarse.hip
    const float *y = Q + (size_t)q * D.d, *row = D.centroids + (size_t)c * D.d;
    double acc = 0.0;
    if (metric == 0) {
      for (int j = 0; j < D.d; ++j) {
        const double t = (double)y[j] - (double)row[j];
        acc = __builtin_fma(t, t, acc);
      }
    } else {
      for (int j = 0; j < D.d; ++j) acc = __builtin_fma((double)y[j], (double)row[j], acc);
    }
    return acc;
  };
  auto key_of_score = [&](double x) -> uint64_t {
    x = (metric == 0 ? x : -x) + 0.0;  // +0.0 folds -0 into +0
    return key_of_double(x);
  };
  bool done = false;  // k1 / k2 / pay hold the nprobe winners, not yet sorted
  if (FROM_APPROX && nprobe < n) {
    const float *ap = S.approx + (size_t)q * n;
    // |y|^2 for the error band
    float yn = 0.f;
    for (int j = threadIdx.x; j < D.d; j += kSelThreads) { const float v = Q[(size_t)q * D.d + j]; yn = fmaf(v, v, yn); }
    for (int o = kWave / 2; o > 0; o >>= 1) yn += __shfl_xor(yn, o);
    if ((threadIdx.x & (kWave - 1)) == 0) s_red[threadIdx.x / kWave] = yn;
    __syncthreads();
    yn = 0.f;
    for (int w = 0; w < kSelThreads / kWave; ++w) yn += s_red[w];
    const float cmax = __uint_as_float(D.ctrl->cnorm_max_bits);
    const float band = 8.f * (float)(D.d + 4) * 5.9604645e-8f * (yn + cmax) * 1.01f;  // 2 E, see coarse_mfma.hip
    const SelectResult ra = wg_radix_select<32>(
        n, (uint32_t)nprobe, [&](int i, uint64_t &k) { k = key_of_float(ap[i] + 0.0f); return true; }, hist, bc);
    const uint32_t tk = (uint32_t)ra.T;  // key of (an upper bound of) the nprobe-th smallest approximation
    const float t = __uint_as_float((tk & 0x80000000u) ? (tk & 0x7fffffffu) : ~tk);
    const float limit = t + band;
    if (threadIdx.x == 0) cnt[0] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += kSelThreads)
      if (ap[i] <= limit) {
        uint32_t p = atomicAdd(&cnt[0], 1u);
        if (p < (uint32_t)kMaxNprobe) pay[p] = (uint32_t)i;
      }
    __syncthreads();
    const int nc = (int)cnt[0];
    if (nc >= nprobe && nc <= kMaxNprobe) {  // (fewer than nprobe: scores that do not compare, e.g. NaN)
      for (int p = threadIdx.x; p < nc; p += kSelThreads) {
        const int c = (int)pay[p];
        k1[p] = key_of_score(exact(c));
        k2[p] = (uint64_t)c;
      }
      wg_sort(nc, k1, k2, pay);  // by (exact score, index): the first nprobe are the answer
      done = true;
    } else {
      for (int i = threadIdx.x; i < n; i += kSelThreads) sc[i] = exact(i);  // the filter did not narrow it: whole row
      __syncthreads();
    }
  }
  auto key1 = [&](int i) -> uint64_t { return key_of_score(sc[i]); };

  SelectResult r1{~0ull, 0, 0}, r2{~0ull, 0, 0};
  const bool all = nprobe >= n;
  if (!done && FROM_APPROX && all) {  // every list is probed: exact order of the whole row
    for (int i = threadIdx.x; i < n; i += kSelThreads) sc[i] = exact(i);
    __syncthreads();
  }
  if (!done) {
  if (!all) {
    r1 = wg_radix_select<64>(n, (uint32_t)nprobe, [&](int i, uint64_t &k) { k = key1(i); return true; },
                             hist, bc);
    if (r1.c_eq > r1.need)  // ties at the boundary go to the lower index
      r2 = wg_radix_select<32>(n, r1.need,
                               [&](int i, uint64_t &k) { k = (uint32_t)i; return key1(i) == r1.T; },
                               hist, bc);
  }
  if (threadIdx.x == 0) cnt[0] = 0;
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += kSelThreads) {
    uint64_t k = key1(i);
    bool take = all || k < r1.T || (k == r1.T && (r1.c_eq <= r1.need || (uint64_t)i <= r2.T));
    if (take) {
      uint32_t p = atomicAdd(&cnt[0], 1u);
      k1[p] = k; k2[p] = (uint64_t)i; pay[p] = (uint32_t)i;
    }
  }
  __syncthreads();
  wg_sort(nprobe, k1, k2, pay);
  }  // !done
  if (done) {  // the sort carried no payload: the list index is the second key
    __syncthreads();
    for (int p = threadIdx.x; p < nprobe; p += kSelThreads) pay[p] = (uint32_t)k2[p];
    __syncthreads();
  }

  // plan
  int32_t *pl = S.probe_list + (size_t)q * max_nprobe;
  uint32_t *plen = S.probe_len + (size_t)q * max_nprobe;
  uint32_t *poff = S.probe_off + (size_t)q * max_nprobe;
  for (int p = threadIdx.x; p < nprobe; p += kSelThreads) {
    int list = (int)pay[p];
    pl[p] = list;
    if (probe_out) probe_out[(size_t)q * nprobe + p] = list;
    uint32_t len = __hip_atomic_load(&D.visible_len[list], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
    plen[p] = len;
    pay[p] = len;  // reuse as lengths for the prefix sum below
    // rank of this pair among the pairs that probe the same list (grouping for the scan)
    S.pair_slot[(size_t)q * max_nprobe + p] = atomicAdd(&S.list_cnt[list], 1u);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long tot = 0;
    for (int p = 0; p < nprobe; ++p) {
      uint32_t len = pay[p];
      poff[p] = (uint32_t)tot;
      tot += len;
    }
    unsigned long long base = 0;
    if (probe_out) tot = 0;  // the probe hook: nothing is scanned afterwards, no room for records is taken
    if (tot > 0xFFFFFFFFull) tot = ~0ull;  // cannot be indexed: treated as overflow below
    if (tot != ~0ull) base = atomicAdd(S.cursor, tot);
    if (tot != ~0ull && base + tot > S.cand_cap) {  // does not fit into the slice any more: the shared reserve
      base = overflow_take(S, tot);
      if (base == ~0ull) tot = ~0ull;
    }
    if (tot == ~0ull) {  // not enough candidate scratch for this query
      base = 0;
      atomicCAS(&D.ctrl->search_error, 0, -6);
      D.mirror->search_error = -6;
      tot = 0;
      for (int p = 0; p < nprobe; ++p) { plen[p] = 0; poff[p] = 0; }
    }
    S.qbase[q] = base;
    S.qtotal[q] = (uint32_t)tot;
  }
}

// ------------------------------------------------------------- pruning bound
// Score of one vector against one query, 4 dimensions at a time, one FMA chain
// in the order of the dimensions.
typedef __attribute__((address_space(1))) float GlobalFloat;
typedef __attribute__((address_space(1))) uint32_t GlobalU32;

template <int METRIC>
__device__ __forceinline__ void accumulate(float &acc, const float4 &x, const float4 &y) {
  if (METRIC == 0) {
    const float t0 = x.x - y.x, t1 = x.y - y.y, t2 = x.z - y.z, t3 = x.w - y.w;
    acc = fmaf(t0, t0, acc); acc = fmaf(t1, t1, acc); acc = fmaf(t2, t2, acc); acc = fmaf(t3, t3, acc);
  } else {
    acc = fmaf(x.x, y.x, acc); acc = fmaf(x.y, y.y, acc); acc = fmaf(x.z, y.z, acc); acc = fmaf(x.w, y.w, acc);
  }
}

constexpr int kGroupThreads = 1024;
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
template <int METRIC, int ST>
__device__ void sample_scores(const Dev &D, int nprobe, int max_nprobe, int q, uint32_t want_groups,
                              const float *__restrict__ Q, const SearchScratch &S, const float4 *qv,
                              uint32_t *skey) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int d4 = D.vchunks;  // 16-byte chunks of a stored vector
  constexpr int kPieces = pieces_of(ST);  // float4s of the query that go with a chunk
  const uint32_t gpb = (uint32_t)D.groups_per_block;
  const size_t group_stride = (size_t)d4 * kWave;
  // the sample is the first want_groups groups of the probed lists taken in order, nearest first
  uint32_t g_first = 0;  // groups of the lists before list p
  for (int p = 0; p < nprobe && g_first < want_groups; ++p) {  // uniform over the workgroup
    const size_t o = (size_t)q * max_nprobe + p;
    const int list = S.probe_list[o];
    const uint32_t len = S.probe_len[o];
    uint32_t groups = (len + kWave - 1) / kWave;
    const uint32_t have = D.nblk[list] * gpb;  // never index the block table past the chain
    if (groups > have) groups = have;
    if (groups > want_groups - g_first) groups = want_groups - g_first;
    for (uint32_t g = (uint32_t)wave; g < groups; g += kGroupThreads / kWave) {
      const uint32_t b = (uint32_t)*table_entry(D, list, g / gpb);
      const float4 *__restrict__ x = block_vecs(D, b) + (size_t)(g % gpb) * group_stride + lane;
      float acc = 0.f;
      int c = 0;
      for (; c + 8 <= d4; c += 8) {  // eight loads of 1 KiB in flight per wavefront
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
    for (uint32_t g = (uint32_t)wave; g < groups; g += kGroupThreads / kWave) {
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

template <bool PQ>
__device__ void sample_bound(const Dev &D, int q, int nprobe, int max_nprobe, int k, const float *__restrict__ Q,
                             const SearchScratch &S) {
  __shared__ float4 qv[512];  // the query (d <= 2048)
  __shared__ uint32_t skey[kSampleMax];
  __shared__ __attribute__((aligned(8))) uint32_t hist[256];
  __shared__ uint32_t bc[4];
  const int tid = threadIdx.x;
  // A query with no more candidates than the selection holds in LDS at once needs no bound.  For
  // inner products neither does one whose records cost less than a sample would: the sample is 512
  // vectors or more read by one workgroup (80 us at d = 768), a record is 8 bytes (short lists, wide
  // vectors).  (For L2 the bound also lets the scan stop early, which is worth the sample.)
  const uint32_t no_bound_below =
      D.metric == 0 ? (uint32_t)kNoBoundBelow : max((uint32_t)kNoBoundBelow, 32u * (uint32_t)D.d);
  if (S.qtotal[q] <= no_bound_below) {  // uniform over the workgroup
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
  const uint32_t part = S.probe_len[(size_t)q * max_nprobe] / (uint32_t)kSampleDivisor;
  want = want < part ? part : want;
  want = want < 512u ? 512u : (want > cap ? cap : want);
  const uint32_t want_groups = (want + kWave - 1) / kWave;
  if (!PQ)
    for (int c = tid; c < D.d4; c += kGroupThreads) qv[c] = reinterpret_cast<const float4 *>(Q + (size_t)q * D.d)[c];
  for (int i = tid; i < (int)(want_groups * kWave); i += kGroupThreads) skey[i] = 0xFFFFFFFFu;
  __syncthreads();
  if (PQ) pq_sample_scores(D, nprobe, max_nprobe, q, want_groups, S, skey);
  else if (D.metric == 0) {
    if (D.storage == 1) sample_scores<0, 1>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey);
    else if (D.storage == 2) sample_scores<0, 2>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey);
    else sample_scores<0, 0>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey);
  } else {
    if (D.storage == 1) sample_scores<1, 1>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey);
    else if (D.storage == 2) sample_scores<1, 2>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey);
    else sample_scores<1, 0>(D, nprobe, max_nprobe, q, want_groups, Q, S, qv, skey);
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
    S.bound[q] = bound;
    S.rec_cnt[q] = 0u;
  }
}

// ------------------------------------------------------------ pair grouping
// The (query, probed list) pairs of a request are grouped by list, so that the
// scan reads a list once for up to kScanTileQueries queries.  One workgroup:
// prefix sums over the lists of the pair counts, the work-item counts and the
// work, then the item descriptors, the split of the items over the 8 XCDs and
// the grouped pair array.  A work item is (list, segment of seg_groups
// 64-vector groups, tile of up to kScanTileQueries of the queries probing the
// list); one wavefront walks it.  The items of one segment follow each other, so
// they run at the same time on the same CU or on its neighbours and the segment
// comes from HBM once.  Segments bound the work of one item, so that long lists
// spread over many wavefronts.  The segment length is the shortest power of two
// for which the request has at most `item_budget` items and no XCD more than
// `max_per_xcd` (the launch of the scan is sized from those two).
constexpr int kSegChoices = 8;  // segment lengths 2, 4, ..., 256 groups
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
// running sum of the pair counts over the lists, 1024 consecutive lists at a time, 16 rows in flight).
__device__ void scatter_pairs(const Dev &D, int nq, int nprobe, int max_nprobe, const SearchScratch &S) {
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
  const int npairs = nq * nprobe;
  for (int base = tid; base < npairs; base += 8 * kGroupThreads) {
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

__global__ __launch_bounds__(kGroupThreads) void k_group(Dev D, int nq, int nprobe, int max_nprobe, int k,
                                                         const float *__restrict__ Q,
                                                         uint32_t item_budget, uint32_t max_per_xcd,
                                                         SearchScratch S) {
  if (blockIdx.x == 1) {  // uniform over the workgroup: this one groups the pairs by list
    scatter_pairs(D, nq, nprobe, max_nprobe, S);
    return;
  }
  if (blockIdx.x > 1) {  // this one sets the bound of query blockIdx.x - 2
    sample_bound<false>(D, (int)blockIdx.x - 2, nprobe, max_nprobe, k, Q, S);
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
  uint4 *__restrict__ plist = S.plist;
  uint32_t *__restrict__ pistart = S.pistart;
  ScanQueues *Qs = S.queues;
  // Cost of a list for the split over the XCDs, per group of 64 vectors: reading it once from HBM
  // (each XCD has its own link to memory) plus the arithmetic of every query that probes it.  On
  // this chip one group's bytes cost about as much as the arithmetic of 12 queries (L2) or 24 (IP).
  const uint32_t byte_weight = D.metric == 0 ? 12u : 24u;

  // The probed lists, compacted in list order (neighbouring lists sit in neighbouring blocks after a
  // bulk load, and the scan reads faster in that order): entry = {list, first pair, pairs, length}.
  // The pair counters are read 1024 consecutive lists at a time, 16 such rows per thread in flight;
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
      const uint32_t tiles = (c[t] + kScanTileQueries - 1) / kScanTileQueries;
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
  // that the loads of a chunk go out together: this workgroup is alone on its CU, and a pass over the
  // entries is a chain of memory latencies otherwise.
  const uint32_t per = (n_c + kGroupThreads - 1) / kGroupThreads;
  const uint32_t e0 = min(n_c, (uint32_t)tid * per), e1 = min(n_c, e0 + per);
  __syncthreads();
  int choice = kSegChoices - 1;
  for (int e = 0; e < kSegChoices; ++e)
    if (s_items[e] <= item_budget && s_items[e] <= S.item_cap) { choice = e; break; }

  for (;; ++choice) {  // uniform: every thread sees the same totals
    const uint32_t seg = 2u << choice;
    uint32_t np = 0, ni = 0;
    unsigned long long wk = 0;
    for (uint32_t eb = e0; eb < e1; eb += kListChunk) {
      uint4 pl[kListChunk];
#pragma unroll
      for (int t = 0; t < kListChunk; ++t) pl[t] = eb + t < e1 ? plist[eb + t] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int t = 0; t < kListChunk; ++t) {
        const uint32_t c = pl[t].z;
        if (!c) continue;
        const uint32_t groups = (pl[t].w + kWave - 1) / kWave;
        np += c;
        ni += (groups ? (groups + seg - 1) / seg : 1u) * ((c + kScanTileQueries - 1) / kScanTileQueries);
        wk += (unsigned long long)(c + byte_weight) * (groups ? groups : 1u);
      }
    }
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
      for (uint32_t eb = e0; eb < e1; eb += kListChunk) {
        uint4 pl[kListChunk];
#pragma unroll
        for (int t = 0; t < kListChunk; ++t) pl[t] = eb + t < e1 ? plist[eb + t] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int t = 0; t < kListChunk; ++t) {
          const uint32_t c = pl[t].z;
          if (!c) continue;
          const uint32_t groups = (pl[t].w + kWave - 1) / kWave;
          const unsigned long long w = (unsigned long long)(c + byte_weight) * (groups ? groups : 1u);
          const uint32_t n =
              (groups ? (groups + seg - 1) / seg : 1u) * ((c + kScanTileQueries - 1) / kScanTileQueries);
          for (uint32_t x = 1; x < 8; ++x) {  // the cut falls inside this list: at the item the same share of it ends at
            const unsigned long long cut = total_work * x / 8;
            if (ws <= cut && cut < ws + w) s_begin[x] = is + (uint32_t)((cut - ws) * n / w);
          }
          is += n;
          ws += w;
        }
      }
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
      for (uint32_t eb = e0; eb < e1; eb += kListChunk) {
        uint4 pl[kListChunk];
#pragma unroll
        for (int t = 0; t < kListChunk; ++t) pl[t] = eb + t < e1 ? plist[eb + t] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int t = 0; t < kListChunk; ++t) {
          const uint32_t c = pl[t].z;
          if (!c) continue;
          const uint32_t groups = (pl[t].w + kWave - 1) / kWave;
          plist[eb + t] = make_uint4(pl[t].x, ps, c, pl[t].w);
          pistart[eb + t] = is;
          ps += c;
          is += (groups ? (groups + seg - 1) / seg : 1u) * ((c + kScanTileQueries - 1) / kScanTileQueries);
        }
      }
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
          tiles = (pl.z + kScanTileQueries - 1) / kScanTileQueries;
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
        const uint32_t tiles = (pl.z + kScanTileQueries - 1) / kScanTileQueries;
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

// ------------------------------------------------------------------ list scan
// A work item is one segment of one list; it is walked once per tile of up to
// kScanTileQueries of the queries that probe the list.  Every WAVEFRONT works on its own: it
// takes an item from a queue, copies the item's queries into its slice of LDS,
// and walks the segment in pairs of groups of 64 vectors, lane = vector (two
// vectors per lane).  Per chunk of 4 dimensions it loads 1 KiB of consecutive
// memory per group (one float4 per lane) ONCE and every lane accumulates the
// score of its two vectors against each query of the item; a query chunk is one
// broadcast LDS read shared by both vectors.  Scores go to each query's
// candidate slice.  No workgroup barrier is involved anywhere.

// Chunks of 4 dimensions per register set of the software pipeline.  Deeper sets for
// items with few queries were measured: they cost a wavefront of occupancy and gain nothing.
constexpr int prefetch_chunks(int) { return 2; }

template <int METRIC, int NQ, int ST>
__device__ __forceinline__ void scan_item(const Dev &D, const SearchScratch &S,
                                          const float *__restrict__ Q, int max_nprobe, int list,
                                          uint32_t first, uint32_t g_begin, uint32_t g_count,
                                          float4 *qs) {
  constexpr int kPrefetch = prefetch_chunks(NQ);
  // Partial-distance pruning (L2 only: squared distances only grow) pays for tiles of few queries,
  // where whole pairs of groups drop out; with more queries somebody is nearly always still in
  // and the branches cost more than the skipped arithmetic saves (measured: 8 queries 3 % slower).
  constexpr bool kPrune = METRIC == 0 && NQ <= 4;
  // Narrow storage: a 16-byte chunk of a stored vector holds 8 halves or 16 bytes, i.e. kPieces
  // float4s' worth of dimensions; they are widened in registers, piece by piece, and meet the
  // matching float4 of each query.  vc chunks per stored vector, d4 float4s per query.
  constexpr int kPieces = pieces_of(ST);
  const int d4 = D.d4, vc = D.vchunks;
  const int lane = threadIdx.x & (kWave - 1);
  // lane i < NQ looks after query i of the item: how far its list goes, its bound, where its
  // survivor records go
  uint32_t my_q = 0, my_len = 0, my_off = 0, my_bound = 0;
  uint64_t my_keys = 0, my_poss = 0;  // addresses of the query's survivor records (keys, positions)
  if (lane < NQ) {
    const uint32_t pk = S.grouped[first + lane];
    my_q = pk >> 10;
    const size_t o = (size_t)my_q * max_nprobe + (pk & 1023u);
    my_len = S.probe_len[o];
    my_off = S.probe_off[o];
    const unsigned long long qb = S.qbase[my_q];
    my_keys = (uint64_t)(uintptr_t)rec_keys_of(S, qb);
    my_poss = (uint64_t)(uintptr_t)rec_poss_of(S, qb);
    my_bound = S.bound[my_q];
  }
  // the bound as a score (L2: keys of non-negative floats order like the floats; "keep everything" is +inf)
  const uint32_t my_boundf = my_bound == 0xFFFFFFFFu ? 0x7F800000u : (my_bound & 0x7FFFFFFFu);
  uint32_t maxlen = 0;
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const uint32_t q = (uint32_t)__builtin_amdgcn_readlane((int)my_q, i);
    const uint32_t len = (uint32_t)__builtin_amdgcn_readlane((int)my_len, i);
    maxlen = len > maxlen ? len : maxlen;
    const float4 *src = reinterpret_cast<const float4 *>(Q + (size_t)q * D.d);
    for (int c = lane; c < d4; c += kWave) qs[i * d4 + c] = src[c];
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();

  uint32_t ngroups = (maxlen + kWave - 1) / kWave;  // groups any query of the item wants
  if (ngroups > g_begin + g_count) ngroups = g_begin + g_count;  // ... inside this item's segment
  const uint32_t gpb = (uint32_t)D.groups_per_block;
  {  // never index the block table past the list's chain, whatever the descriptors say
    const uint32_t have = D.nblk[list] * gpb;
    if (ngroups > have) ngroups = have;
  }
  const size_t group_stride = (size_t)vc * kWave;
  for (uint32_t g0 = g_begin; g0 < ngroups; g0 += 2) {
    const bool two = g0 + 1 < ngroups;  // uniform over the wavefront
    const uint32_t g1 = two ? g0 + 1 : g0;
    const uint32_t b0 = (uint32_t)*table_entry(D, list, g0 / gpb);
    const uint32_t b1 = (uint32_t)*table_entry(D, list, g1 / gpb);
    const float4 *__restrict__ xa = block_vecs(D, b0) + (size_t)(g0 % gpb) * group_stride + lane;
    const float4 *__restrict__ xb = block_vecs(D, b1) + (size_t)(g1 % gpb) * group_stride + lane;
    float acc0[NQ], acc1[NQ];
#pragma unroll
    for (int i = 0; i < NQ; ++i) { acc0[i] = 0.f; acc1[i] = 0.f; }
    uint32_t alive = (1u << NQ) - 1u;  // queries of the item that can still keep a vector of this pair of groups
    const uint32_t v0 = g0 * kWave + lane, v1 = v0 + kWave;
    // Software pipeline over the chunks, two register sets of kPrefetch chunks
    // each: while one set is being accumulated the loads of the other are in
    // flight.
    const int d4_main = vc & ~(2 * kPrefetch - 1);
    if (d4_main) {
      float4 a0[kPrefetch], a1[kPrefetch], b0v[kPrefetch], b1v[kPrefetch];
      auto load_set = [&](float4 *s0, float4 *s1, int cb) {
#pragma unroll
        for (int u = 0; u < kPrefetch; ++u) {
          s0[u] = xa[(size_t)(cb + u) * kWave];
          s1[u] = xb[(size_t)(cb + u) * kWave];
        }
        __builtin_amdgcn_sched_barrier(0);  // loads are issued here, not sunk towards their use
      };
      auto use_set = [&](const float4 *s0, const float4 *s1, int cb) {
        if (ST == 0) {
#pragma unroll
          for (int i = 0; i < NQ; ++i) {
            if (kPrune && !((alive >> i) & 1u)) continue;  // uniform: this query is out for this pair of groups
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u) {
              const float4 y = qs[i * d4 + cb + u];
              accumulate<METRIC>(acc0[i], s0[u], y);
              accumulate<METRIC>(acc1[i], s1[u], y);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep one query's temporaries from piling up on the next
          }
        } else {
#pragma unroll
          for (int u = 0; u < kPrefetch; ++u) {
#pragma unroll
            for (int s = 0; s < kPieces; ++s) {
              const float4 x0 = chunk_piece<ST>(s0[u], s), x1 = chunk_piece<ST>(s1[u], s);
#pragma unroll
              for (int i = 0; i < NQ; ++i) {
                if (kPrune && !((alive >> i) & 1u)) continue;  // uniform
                const float4 y = qs[i * d4 + (cb + u) * kPieces + s];
                accumulate<METRIC>(acc0[i], x0, y);
                accumulate<METRIC>(acc1[i], x1, y);
              }
              __builtin_amdgcn_sched_barrier(0);  // one piece's widened values at a time
            }
          }
        }
      };
      load_set(a0, a1, 0);
      int c = 0;
#pragma unroll 1
      for (; c + 2 * kPrefetch < d4_main; c += 2 * kPrefetch) {
        load_set(b0v, b1v, c + kPrefetch);
        use_set(a0, a1, c);
        load_set(a0, a1, c + 2 * kPrefetch);
        use_set(b0v, b1v, c + kPrefetch);
        if (kPrune) {
          // Squared distances only grow: a query none of whose 128 vectors can still come in under
          // its bound takes no further part in this pair of groups, and when no query is left the
          // rest of the pair is not read.
#pragma unroll
          for (int i = 0; i < NQ; ++i) {
            if (!((alive >> i) & 1u)) continue;
            const uint32_t len = (uint32_t)__builtin_amdgcn_readlane((int)my_len, i);
            const float bf = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)my_boundf, i));
            const bool live = (v0 < len && !(acc0[i] > bf)) || (two && v1 < len && !(acc1[i] > bf));
            if (__ballot(live) == 0ull) alive &= ~(1u << i);
          }
          if (alive == 0u) break;
        }
      }
      if (alive != 0u) {
        load_set(b0v, b1v, c + kPrefetch);
        use_set(a0, a1, c);
        use_set(b0v, b1v, c + kPrefetch);
      }
    }
    for (int c = d4_main; c < vc && alive != 0u; ++c) {  // chunks beyond the last full double set
      const float4 r0 = xa[(size_t)c * kWave], r1 = xb[(size_t)c * kWave];
#pragma unroll
      for (int s = 0; s < kPieces; ++s) {
        const float4 x0 = chunk_piece<ST>(r0, s), x1 = chunk_piece<ST>(r1, s);
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
          const float4 y = qs[i * d4 + c * kPieces + s];
          accumulate<METRIC>(acc0[i], x0, y);
          accumulate<METRIC>(acc1[i], x1, y);
        }
      }
    }
    // Only what is not worse than the query's bound is kept: appended to the query's survivor
    // records, one atomic per query with survivors.  (readlane yields a signed int: go through
    // uint32_t so the low word is not sign-extended.  A pointer rebuilt from integers has no address
    // space: say "global", or the stores become FLAT operations, and while one of those is pending
    // every wait of the load pipeline above has to be for ALL outstanding memory operations.)
    auto lane_u32 = [](uint32_t v, int i) { return (uint32_t)__builtin_amdgcn_readlane((int)v, i); };
    auto lane_u64 = [&](uint64_t v, int i) {
      return (uint64_t)lane_u32((uint32_t)v, i) | ((uint64_t)lane_u32((uint32_t)(v >> 32), i) << 32);
    };
    {
      // survivors of each query in this pair of groups: masks, counts (lane i keeps query i's count)
      unsigned long long m0[NQ], m1[NQ];
      uint32_t n_mine = 0;
      bool any = false;
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        const uint32_t len = lane_u32(my_len, i), bound = lane_u32(my_bound, i);
        const uint32_t key0 = key_of_float((METRIC == 0 ? acc0[i] : -acc0[i]) + 0.0f);
        const uint32_t key1 = key_of_float((METRIC == 0 ? acc1[i] : -acc1[i]) + 0.0f);
        m0[i] = __ballot(v0 < len && key0 <= bound);
        m1[i] = __ballot(two && v1 < len && key1 <= bound);
        const uint32_t c = (uint32_t)__popcll(m0[i]) + (uint32_t)__popcll(m1[i]);
        n_mine = lane == i ? c : n_mine;
        any = any || c != 0;
      }
      if (any) {  // uniform.  One atomic per query with survivors, all of them in one instruction
        uint32_t base_mine = 0;
        if (lane < NQ && n_mine) base_mine = atomicAdd(&S.rec_cnt[my_q], n_mine);
        const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
          if ((m0[i] | m1[i]) == 0) continue;  // uniform
          const uint64_t at = 4ull * lane_u32(base_mine, i);
          const uint32_t off = lane_u32(my_off, i);
          GlobalU32 *rk = (GlobalU32 *)(lane_u64(my_keys, i) + at);
          GlobalU32 *rp = (GlobalU32 *)(lane_u64(my_poss, i) + at);
          if ((m0[i] >> lane) & 1ull) {
            const uint32_t slot = (uint32_t)__popcll(m0[i] & below);
            rk[slot] = key_of_float((METRIC == 0 ? acc0[i] : -acc0[i]) + 0.0f);
            rp[slot] = off + v0;
          }
          if ((m1[i] >> lane) & 1ull) {
            const uint32_t slot = (uint32_t)__popcll(m0[i]) + (uint32_t)__popcll(m1[i] & below);
            rk[slot] = key_of_float((METRIC == 0 ? acc1[i] : -acc1[i]) + 0.0f);
            rp[slot] = off + v1;
          }
        }
      }
    }
  }
  __builtin_amdgcn_wave_barrier();  // the LDS slice is rewritten by the next item
}

// The hardware's workgroup dispatcher is the work queue (a new workgroup starts
// wherever room frees up).  A workgroup is four wavefronts that take four
// consecutive work items, one each, and work on their own: own slice of LDS, no
// barrier.  Consecutive items are mostly the tiles of one segment, or the next
// segment of the same list.  Hardware hands consecutive workgroup ids to the 8
// XCDs in turn, so workgroup i runs on XCD i % 8 and takes items 4 (i / 8) ..
// 4 (i / 8) + 3 of that XCD's range of items (a contiguous range of lists).
// Wavefronts past the end of their range leave at once.
constexpr uint32_t kXcds = 8;
constexpr int kScanWaves = 4;

template <int METRIC, int ST>
__global__ __launch_bounds__(kScanWaves * kWave) void k_scan(Dev D, int max_nprobe,
                                                             const float *__restrict__ Q, SearchScratch S) {
  extern __shared__ float4 qs_all[];  // [wavefronts][kScanTileQueries][d / 4]
  const ScanQueues *Qs = S.queues;
  const uint32_t x = blockIdx.x % kXcds;
  const uint32_t wave = threadIdx.x / kWave, waves = blockDim.x / kWave;
  const uint32_t item = Qs->begin[x] + (blockIdx.x / kXcds) * waves + wave;
  if (item >= Qs->begin[x + 1]) return;
  const uint32_t seg = Qs->seg_groups;
  if (seg == 0) return;
  float4 *qs = qs_all + (size_t)wave * kScanTileQueries * D.d4;
  const uint4 desc = S.tile_desc[item];
  const int list = __builtin_amdgcn_readfirstlane((int)desc.x);
  const uint32_t first = (uint32_t)__builtin_amdgcn_readfirstlane((int)desc.y);
  const uint32_t pairs = (uint32_t)__builtin_amdgcn_readfirstlane((int)desc.z);
  const uint32_t g_begin = (uint32_t)__builtin_amdgcn_readfirstlane((int)desc.w) * seg;
  switch (pairs) {
    case 0: break;
    case 1: scan_item<METRIC, 1, ST>(D, S, Q, max_nprobe, list, first, g_begin, seg, qs); break;
    case 2: scan_item<METRIC, 2, ST>(D, S, Q, max_nprobe, list, first, g_begin, seg, qs); break;
    case 3: scan_item<METRIC, 3, ST>(D, S, Q, max_nprobe, list, first, g_begin, seg, qs); break;
    case 4: scan_item<METRIC, 4, ST>(D, S, Q, max_nprobe, list, first, g_begin, seg, qs); break;
    case 5: scan_item<METRIC, 5, ST>(D, S, Q, max_nprobe, list, first, g_begin, seg, qs); break;
    case 6: scan_item<METRIC, 6, ST>(D, S, Q, max_nprobe, list, first, g_begin, seg, qs); break;
    case 7: scan_item<METRIC, 7, ST>(D, S, Q, max_nprobe, list, first, g_begin, seg, qs); break;
    default: scan_item<METRIC, 8, ST>(D, S, Q, max_nprobe, list, first, g_begin, seg, qs); break;
  }
}

// ------------------------------------------------- scan of quantised lists
// Product-quantised lists are scanned per QUERY, not per list: what a query brings to a list is
// its table of sub-scores (M x 256 floats, 1 KiB per sub-space, computed once per request), far
// more than the 64 bytes per sub-space of a group of 64 coded vectors, so the table is what has
// to stay put.  Workgroup (q, part) copies the table of query q into LDS once and its wavefronts
// walk part `part` of the groups of the query's probed lists, four groups of 64 vectors at a time,
// lane = vector: per word of 4 codes one coalesced 256-byte load per group and four LDS look-ups
// per vector, added up in the order of the sub-spaces.  (The codes of a probed list are read by
// every query that probes it; they are a small fraction of the flat vectors and stay in cache.)
// Survivors of the query's bound are appended to its records exactly as in the scan of flat lists.
constexpr int kPqScanWaves = 8;

constexpr int kPqScanThreads = kPqScanWaves * kWave;
constexpr int kPqUnits = 4;  // groups of 64 vectors a wavefront walks side by side
constexpr int kPqStage = 128;  // survivors a wavefront collects in LDS before it appends them to the query's records

__device__ inline void pq_flush(const SearchScratch &S, int q, unsigned long long base, const uint32_t *my_key,
                                const uint32_t *my_pos, uint32_t n, int lane) {
  uint32_t at = 0;
  if (lane == 0) at = atomicAdd(&S.rec_cnt[q], n);
  at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
  uint32_t *rk = rec_keys_of(S, base) + at, *rp = rec_poss_of(S, base) + at;
  for (uint32_t i = (uint32_t)lane; i < n; i += kWave) {
    rk[i] = my_key[i];
    rp[i] = my_pos[i];
  }
}

__global__ __launch_bounds__(kPqScanThreads) void k_pq_scan(Dev D, int nprobe, int max_nprobe, int parts,
                                                            SearchScratch S) {
  extern __shared__ float pq_lut[];            // [M][256]
  __shared__ uint32_t gstart[kMaxNprobe + 1];  // groups of the query in front of probe p
  __shared__ uint32_t s_blk[kPqScanThreads];   // per group of the current chunk: its block ...
  __shared__ uint32_t s_probe[kPqScanThreads]; // ... and the probe it belongs to
  __shared__ uint32_t s_key[kPqScanWaves][kPqStage];  // survivors not yet written out, per wavefront
  __shared__ uint32_t s_pos[kPqScanWaves][kPqStage];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int q = blockIdx.x / parts, part = blockIdx.x % parts;
  const int M = D.pq_m, words = M / 4;
  const uint32_t gpb = (uint32_t)D.groups_per_block;
  if (wave == 0) {  // running sum of the groups per probe, 64 probes at a time
    uint32_t carry = 0;
    for (int p0 = 0; p0 < nprobe; p0 += kWave) {
      const int p = p0 + lane;
      uint32_t groups = 0;
      if (p < nprobe) {
        const size_t o = (size_t)q * max_nprobe + p;
        groups = (S.probe_len[o] + kWave - 1) / kWave;
        const uint32_t have = D.nblk[S.probe_list[o]] * gpb;  // never index the block table past the chain
        groups = groups > have ? have : groups;
      }
      uint32_t incl = groups;
      for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
      }
      if (p < nprobe) gstart[p] = carry + incl - groups;
      carry += __shfl(incl, kWave - 1);
    }
    if (lane == 0) gstart[nprobe] = carry;
  }
  __syncthreads();
  const uint32_t total = gstart[nprobe];
  uint32_t per = (total + (uint32_t)parts - 1) / (uint32_t)parts;
  const uint32_t u_lo = (uint32_t)part * per, u_hi = min(total, u_lo + per);
  if (u_lo >= u_hi) return;  // uniform over the workgroup
  // the query's table: loads issued here, stored to LDS after the first chunk's blocks are resolved
  constexpr int kLutRegs = 64 * 64 / kPqScanThreads;  // float4 per thread at M = 64
  float4 lut_reg[kLutRegs];
  {
    const float4 *src = reinterpret_cast<const float4 *>(S.lut + (size_t)q * M * 256);
#pragma unroll
    for (int r = 0; r < kLutRegs; ++r) {
      const int i = tid + r * kPqScanThreads;
      lut_reg[r] = i < M * 64 ? src[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  const unsigned long long base = S.qbase[q];
  const uint32_t bound = __hip_atomic_load(&S.bound[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const int metric = D.metric;
  uint32_t *my_key = s_key[wave], *my_pos = s_pos[wave];
  uint32_t staged = 0;  // uniform over the wavefront
  for (uint32_t c0 = u_lo; c0 < u_hi; c0 += kPqScanThreads) {  // chunks of 512 groups
    if (c0 != u_lo) __syncthreads();  // the previous chunk has been walked
    {  // thread t resolves group c0 + t: probe by bisection of the running sums, block from the list's table
      const uint32_t u = c0 + (uint32_t)tid;
      if (u < u_hi) {
        int lo = 0, hi = nprobe - 1;  // last probe whose groups start at or before u
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (gstart[mid] <= u) lo = mid; else hi = mid - 1;
        }
        const int list = S.probe_list[(size_t)q * max_nprobe + lo];
        s_probe[tid] = (uint32_t)lo;
        s_blk[tid] = (uint32_t)*table_entry(D, list, (u - gstart[lo]) / gpb);
      }
    }
    if (c0 == u_lo) {
      float4 *dst = reinterpret_cast<float4 *>(pq_lut);
#pragma unroll
      for (int r = 0; r < kLutRegs; ++r) {
        const int i = tid + r * kPqScanThreads;
        if (i < M * 64) dst[i] = lut_reg[r];
      }
    }
    __syncthreads();
    const uint32_t n_here = min((uint32_t)kPqScanThreads, u_hi - c0);
    // a wavefront takes kPqUnits consecutive groups at a time: all their loads are in flight together,
    // and their survivors are appended with one reservation
    for (uint32_t i0 = (uint32_t)(kPqUnits * wave); i0 < n_here; i0 += kPqUnits * kPqScanWaves) {
      const uint32_t *__restrict__ x[kPqUnits];
      uint32_t len[kPqUnits], off[kPqUnits], v[kPqUnits];
      bool live[kPqUnits];
#pragma unroll
      for (int j = 0; j < kPqUnits; ++j) {
        live[j] = i0 + j < n_here;  // uniform over the wavefront
        const uint32_t i = live[j] ? i0 + j : i0;
        // the same for every lane: kept in scalar registers, so is the address arithmetic below
        const uint32_t p = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_probe[i]);
        const uint32_t blk = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_blk[i]);
        const uint32_t g = c0 + i - (uint32_t)__builtin_amdgcn_readfirstlane((int)gstart[p]);
        const size_t o = (size_t)q * max_nprobe + p;
        x[j] = block_codes(D, blk) + (size_t)(g % gpb) * words * kWave + lane;
        len[j] = S.probe_len[o];
        off[j] = S.probe_off[o];
        v[j] = g * kWave + lane;
      }
      float acc[kPqUnits];
#pragma unroll
      for (int j = 0; j < kPqUnits; ++j) acc[j] = 0.f;
      for (int cw = 0; cw < words; cw += 4) {  // 16 codes of every group at a time: their loads go out together
        uint32_t w[4][kPqUnits];
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
#pragma unroll
          for (int j = 0; j < kPqUnits; ++j) w[cc][j] = cw + cc < words ? x[j][(size_t)(cw + cc) * kWave] : 0u;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
          if (cw + cc < words) {  // uniform
            const float *t = pq_lut + (size_t)(cw + cc) * 4 * 256;
#pragma unroll
            for (int j = 0; j < kPqUnits; ++j) acc[j] += t[w[cc][j] & 255u];
#pragma unroll
            for (int j = 0; j < kPqUnits; ++j) acc[j] += t[256 + ((w[cc][j] >> 8) & 255u)];
#pragma unroll
            for (int j = 0; j < kPqUnits; ++j) acc[j] += t[512 + ((w[cc][j] >> 16) & 255u)];
#pragma unroll
            for (int j = 0; j < kPqUnits; ++j) acc[j] += t[768 + (w[cc][j] >> 24)];
          }
        }
      }
      uint32_t key[kPqUnits];
      unsigned long long mask[kPqUnits];
      uint32_t n_keep = 0;
#pragma unroll
      for (int j = 0; j < kPqUnits; ++j) {
        key[j] = key_of_float((metric == 0 ? acc[j] : -acc[j]) + 0.0f);
        mask[j] = __ballot(live[j] && v[j] < len[j] && key[j] <= bound);
        n_keep += (uint32_t)__popcll(mask[j]);
      }
      // Survivors wait in the wavefront's own slice of LDS and go out kPqStage at a time: every
      // reservation of a query goes to the same word, so the fewer the better.
      if (staged + n_keep > (uint32_t)kPqStage) {  // uniform over the wavefront
        pq_flush(S, q, base, my_key, my_pos, staged, lane);
        staged = 0;
      }
      if (n_keep > (uint32_t)kPqStage) {  // more than the slice holds: straight out
        uint32_t at = 0;
        if (lane == 0) at = atomicAdd(&S.rec_cnt[q], n_keep);
        at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
        const unsigned long long below = (1ull << lane) - 1ull;
        uint32_t *rk = rec_keys_of(S, base) + at, *rp = rec_poss_of(S, base) + at;
#pragma unroll
        for (int j = 0; j < kPqUnits; ++j) {
          if ((mask[j] >> lane) & 1ull) {
            const uint32_t slot = (uint32_t)__popcll(mask[j] & below);
            rk[slot] = key[j];
            rp[slot] = off[j] + v[j];
          }
          rk += __popcll(mask[j]);
          rp += __popcll(mask[j]);
        }
      } else if (n_keep) {
        const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
        for (int j = 0; j < kPqUnits; ++j) {
          if ((mask[j] >> lane) & 1ull) {
            const uint32_t slot = staged + (uint32_t)__popcll(mask[j] & below);
            my_key[slot] = key[j];
            my_pos[slot] = off[j] + v[j];
          }
          staged += (uint32_t)__popcll(mask[j]);
        }
      }
    }
  }
  if (staged) pq_flush(S, q, base, my_key, my_pos, staged, lane);
}

// The bound of every query of a request over quantised lists (the grouping by list that the scan
// of flat lists needs is not made).
// The workgroup of a query first writes the query's table of sub-scores: lut[q][m][c] = squared
// distance (L2) or inner product (IP) between sub-vector m of the query and entry c of codebook m,
// fp32, one FMA chain in the order of the dimensions; its sample and the scan read it from there.
__global__ __launch_bounds__(kGroupThreads) void k_pq_bound(Dev D, int nprobe, int max_nprobe, int k,
                                                            const float *__restrict__ Q, SearchScratch S) {
  const int q = blockIdx.x;
  {
    const int M = D.pq_m, ds = D.d / M;
    const float *__restrict__ yq = Q + (size_t)q * D.d;
    float *__restrict__ lut = S.lut + (size_t)q * M * 256;
    // M * 256 entries, 1024 threads: M / 4 rounds, four of them side by side (their loads overlap);
    // 16-byte loads where the sub-space allows
    for (int i0 = threadIdx.x; i0 < M * 256; i0 += 4 * kGroupThreads) {
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      if (ds % 4 == 0) {  // uniform
        for (int j4 = 0; j4 < ds / 4; ++j4) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int i = i0 + r * kGroupThreads;
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
            const int i = i0 + r * kGroupThreads;
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
        if (i0 + r * kGroupThreads < M * 256) lut[i0 + r * kGroupThreads] = acc[r];
    }
  }
  __threadfence_block();
  __syncthreads();  // the sample below reads the table
  sample_bound<true>(D, q, nprobe, max_nprobe, k, nullptr, S);
}

// ------------------------------------------------------------ top-k selection
// One workgroup per query takes the k best of the query's survivor records
// (what the scan appended for it) by (score, id): exact selection with the id
// tie-break, then a sort of the winners.  The records
// number a few hundred as a rule and are worked on in LDS; a list longer than
// LDS holds (massive ties) is selected from in place.
constexpr int kSurvivorCap = 4096;

constexpr int kTieCap = 1024;  // candidates tied at the k-th score that are told apart in LDS

struct SelectShared {
  __attribute__((aligned(8))) uint32_t hist[256];  // also holds two 64-bit words for a moment
  uint32_t bc[4];
  uint32_t cnt[2];
  uint64_t k1[kMaxK];
  uint64_t k2[kMaxK];
  uint32_t pay[kMaxK];
  uint64_t tie_id[kTieCap];
  uint32_t tie_item[kTieCap];
};

// Exact top-k among `count` items given by key(j) (32-bit score key) and
// item(j) (candidate position, for the id lookup).  Leaves the winners sorted in
// sh.k1 (score key), sh.k2 (id key), sh.pay (candidate position); returns how
// many.  Candidates tied at the k-th score are told apart by id: their ids are
// fetched once and ranked in LDS (with byte-valued data such ties are the rule,
// a handful per query); only more ties than kTieCap go through a radix
// selection over the ids.
template <typename KeyFn, typename ItemFn, typename IdFn>
__device__ int select_topk(int count, int k, KeyFn key, ItemFn item, IdFn id_of, SelectShared &sh) {
  auto key_of_id = [](int64_t id) -> uint64_t { return (uint64_t)id ^ 0x8000000000000000ull; };
  const int kk = k < count ? k : count;
  SelectResult r1{~0ull, 0, 0}, r2{~0ull, 0, 0};
  const bool all = count <= k;
  if (!all)
    r1 = wg_radix_select<32>(count, (uint32_t)k, [&](int j, uint64_t &kv) { kv = key(j); return true; },
                             sh.hist, sh.bc);
  const bool tie_break = !all && r1.c_eq > r1.need;  // not all of the candidates tied at the k-th score fit
  const bool in_lds = tie_break && r1.c_eq <= (uint32_t)kTieCap;
  if (tie_break && !in_lds)
    r2 = wg_radix_select<64>(count, r1.need,
                             [&](int j, uint64_t &kv) {
                               if (key(j) != (uint32_t)r1.T) return false;
                               kv = key_of_id(id_of(item(j)));
                               return true;
                             },
                             sh.hist, sh.bc);
  if (threadIdx.x == 0) sh.cnt[0] = sh.cnt[1] = 0;
  __syncthreads();
  for (int j = threadIdx.x; j < count; j += blockDim.x) {
    const uint32_t kv = key(j);
    bool take = all || kv < (uint32_t)r1.T || (kv == (uint32_t)r1.T && !tie_break);
    int64_t id = 0;
    bool have_id = false;
    if (!take && kv == (uint32_t)r1.T) {
      if (in_lds) {
        sh.tie_item[atomicAdd(&sh.cnt[1], 1u)] = (uint32_t)item(j);
      } else {
        id = id_of(item(j)); have_id = true;
        const uint64_t ik = key_of_id(id);
        if (ik < r2.T) take = true;
        else if (ik == r2.T) take = atomicAdd(&sh.cnt[1], 1u) < r2.need;  // identical (score, id) pairs
      }
    }
    if (take) {
      if (!have_id) id = id_of(item(j));
      const uint32_t p = atomicAdd(&sh.cnt[0], 1u);
      sh.k1[p] = kv; sh.k2[p] = key_of_id(id); sh.pay[p] = (uint32_t)item(j);
    }
  }
  __syncthreads();
  if (in_lds) {  // uniform over the workgroup
    const int nt = (int)sh.cnt[1];  // == r1.c_eq
    for (int t = threadIdx.x; t < nt; t += blockDim.x) sh.tie_id[t] = key_of_id(id_of((int)sh.tie_item[t]));
    __syncthreads();
    for (int t = threadIdx.x; t < nt; t += blockDim.x) {
      const uint64_t mine = sh.tie_id[t];
      uint32_t rank = 0;
      for (int u = 0; u < nt; ++u) {
        const uint64_t other = sh.tie_id[u];
        rank += (other < mine || (other == mine && u < t)) ? 1u : 0u;
      }
      if (rank < r1.need) {
        const uint32_t p = atomicAdd(&sh.cnt[0], 1u);
        sh.k1[p] = (uint32_t)r1.T; sh.k2[p] = mine; sh.pay[p] = sh.tie_item[t];
      }
    }
    __syncthreads();
  }
  wg_sort(kk, sh.k1, sh.k2, sh.pay);
  return kk;
}

constexpr int kTopkThreads = 512;

__device__ inline float score_of_key(uint32_t key, int metric) {
  const float x = __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
  return metric == 0 ? x : -x;
}

__global__ __launch_bounds__(kTopkThreads) void k_select(Dev D, int k, int nprobe, int max_nprobe,
                                                        SearchScratch S, float *__restrict__ out_dist,
                                                        int64_t *__restrict__ out_ids) {
  __shared__ SelectShared sh;
  __shared__ uint32_t offs[kMaxNprobe];
  __shared__ int32_t lists[kMaxNprobe];
  __shared__ uint32_t skey[kSurvivorCap];
  __shared__ uint32_t sidx[kSurvivorCap];
  __shared__ uint32_t scount;
  const int q = blockIdx.x;
  const int n = (int)S.rec_cnt[q];
  const unsigned long long base = S.qbase[q];
  const uint32_t *rk = rec_keys_of(S, base), *rp = rec_poss_of(S, base);
  const int metric = D.metric;
  const int lane = threadIdx.x & (kWave - 1);
  for (int p = threadIdx.x; p < nprobe; p += kTopkThreads) {
    offs[p] = S.probe_off[(size_t)q * max_nprobe + p];
    lists[p] = S.probe_list[(size_t)q * max_nprobe + p];
  }
  if (threadIdx.x == 0) scount = 0;
  __syncthreads();

  // The records are taken into LDS in portions.  Once LDS is more than half full the k-th best
  // of what it holds becomes the limit (it cannot be better than the final k-th best): what is
  // worse is dropped, and later portions are filtered on the way in.  Under a limit only a few
  // per cent of a portion pass as a rule, so a portion is four times what LDS could take if all
  // of it passed; should it not fit after all, what it added is dropped, the limit is renewed
  // and the portion is read again, cut to what fits for certain.  Ties that no limit can
  // separate (LDS stays more than half full) are left to the selection in place below.
  uint32_t limit = S.bound[q];
  bool in_lds = true;
  __shared__ uint32_t s_over;
  int stretch = 1;  // portions as a multiple of the room in LDS
  for (int next = 0; next < n;) {  // every branch here is uniform over the workgroup
    const int count = (int)scount;
    const int m = min(n - next, stretch * (kSurvivorCap - count));
    if (threadIdx.x == 0) s_over = 0;
    __syncthreads();
    constexpr int kInFlight = 8;  // independent loads per thread
    for (int j0 = 0; j0 < m; j0 += kInFlight * kTopkThreads) {
      uint32_t kv[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {  // clamped index: the loads are unconditional and issue back to back
        const int j = j0 + u * kTopkThreads + (int)threadIdx.x;
        kv[u] = rk[next + (j < m ? j : m - 1)];
      }
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {
        const int j = j0 + u * kTopkThreads + (int)threadIdx.x;
        const bool keep = j < m && kv[u] <= limit;
        const unsigned long long mask = __ballot(keep);
        if (mask) {  // uniform over the wavefront
          uint32_t at = 0;
          if (lane == 0) at = atomicAdd(&scount, (uint32_t)__popcll(mask));
          at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
          if (keep) {
            const uint32_t slot = at + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
            if (slot < (uint32_t)kSurvivorCap) { skey[slot] = kv[u]; sidx[slot] = rp[next + j]; }
            else s_over = 1u;
          }
        }
      }
    }
    __syncthreads();
    const bool over = s_over != 0;
    __syncthreads();
    if (over) {  // did not fit: forget what this portion added; below, the limit is renewed from the rest
      if (threadIdx.x == 0) scount = (uint32_t)count;
      __syncthreads();
    } else {
      next += m;
      if (next >= n) break;
    }
    const int have = (int)scount;
    if (!over && have <= kSurvivorCap / 2) continue;
    if (have >= k) {
      // tighten
      const SelectResult r = wg_radix_select<32>(
          have, (uint32_t)k, [&](int j, uint64_t &kv) { kv = skey[j]; return true; }, sh.hist, sh.bc);
      limit = (uint32_t)r.T;
      // drop what is worse: everybody reads its entries, then everybody writes the kept ones back
      constexpr int kMine = kSurvivorCap / kTopkThreads;
      uint32_t mk[kMine], mi[kMine];
#pragma unroll
      for (int u = 0; u < kMine; ++u) {
        const int j = (int)threadIdx.x + u * kTopkThreads;
        mk[u] = j < have ? skey[j] : 0xFFFFFFFFu;
        mi[u] = j < have ? sidx[j] : 0u;
      }
      __syncthreads();
      if (threadIdx.x == 0) scount = 0;
      __syncthreads();
#pragma unroll
      for (int u = 0; u < kMine; ++u) {
        const int j = (int)threadIdx.x + u * kTopkThreads;
        const bool keep = j < have && mk[u] <= limit;
        const unsigned long long mask = __ballot(keep);
        if (mask) {
          uint32_t at = 0;
          if (lane == 0) at = atomicAdd(&scount, (uint32_t)__popcll(mask));
          at = (uint32_t)__builtin_amdgcn_readfirstlane((int)at);
          if (keep) {
            const uint32_t slot = at + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
            skey[slot] = mk[u];
            sidx[slot] = mi[u];
          }
        }
      }
      __syncthreads();
      if ((int)scount > kSurvivorCap / 2) { in_lds = false; break; }
    }
    // from the first limit on, portions may be stretched; a portion that did not fit is read
    // again unstretched (it fits then, whatever it holds)
    stretch = over ? 1 : 4;
  }

  // candidate position -> id: which probed list (last offset <= position), which place, which block
  auto id_of = [&](int i) -> int64_t {
    int lo = 0, hi = nprobe - 1;
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      if (offs[mid] <= (uint32_t)i) lo = mid; else hi = mid - 1;
    }
    uint32_t pos = (uint32_t)i - offs[lo];
    uint32_t b = (uint32_t)*table_entry(D, lists[lo], pos / (uint32_t)D.T_m);
    return block_ids(D, b)[pos % (uint32_t)D.T_m];
  };

  int kk;
  if (in_lds)
    kk = select_topk((int)scount, k, [&](int j) { return skey[j]; }, [&](int j) { return (int)sidx[j]; },
                     id_of, sh);
  else
    kk = select_topk(n, k, [&](int j) { return rk[j]; }, [&](int j) { return (int)rp[j]; }, id_of, sh);

  for (int r = threadIdx.x; r < k; r += kTopkThreads) {
    size_t o = (size_t)q * k + r;
    if (r < kk) {
      out_dist[o] = score_of_key((uint32_t)sh.k1[r], metric);
      out_ids[o] = (int64_t)(sh.k2[r] ^ 0x8000000000000000ull);
    } else {
      out_dist[o] = metric == 0 ? __builtin_inff() : -__builtin_inff();
      out_ids[o] = -1;
    }
  }
  // the records are not looked at any more (the selection ended with a barrier)
  if (threadIdx.x == 0) overflow_request_done(S, gridDim.x);
}

// ---------------------------------------------------------------- launchers

void launch_probe_plan(const Dev &D, int64_t nq, int nprobe, int max_nprobe, const SearchScratch &S,
                       const float *Q, bool from_approx, int32_t *probe_out, hipStream_t s) {
  if (nq <= 0) return;
  if (from_approx)
    hipLaunchKernelGGL(k_probe_plan<true>, dim3((unsigned)nq), dim3(kSelThreads), 0, s, D, nprobe, max_nprobe,
                       S, Q, probe_out);
  else
    hipLaunchKernelGGL(k_probe_plan<false>, dim3((unsigned)nq), dim3(kSelThreads), 0, s, D, nprobe, max_nprobe,
                       S, Q, probe_out);
}

// Wavefronts per workgroup of the scan: as many (4, 2, 1) as fit their query tiles into 64 KiB of LDS
static int scan_waves(const Dev &D) {
  const size_t per_wave = (size_t)kScanTileQueries * D.d * sizeof(float);
  int waves = kScanWaves;
  while (waves > 1 && per_wave * waves > 65536) waves /= 2;
  return waves;
}

// workgroups of the scan launch for a budget of work items (one wavefront each):
// room for an uneven split of the items over the XCDs
static int scan_grid(const Dev &D, int item_budget) {
  const int waves = scan_waves(D);
  const int wgs = (item_budget + item_budget / 2 + waves - 1) / waves;
  return (wgs + (int)kXcds - 1) / (int)kXcds * (int)kXcds;
}

void launch_group(const Dev &D, int64_t nq, int nprobe, int max_nprobe, int k, const float *Q,
                  int item_budget, const SearchScratch &S, hipStream_t s) {
  if (nq <= 0) return;
  if (D.pq_m > 0) {
    hipLaunchKernelGGL(k_pq_bound, dim3((unsigned)nq), dim3(kGroupThreads), 0, s, D, nprobe, max_nprobe, k, Q, S);
    return;
  }
  // workgroup 0 cuts the work items, workgroup 1 groups the pairs, workgroup 2 + q sets the bound of query q
  hipLaunchKernelGGL(k_group, dim3(2 + (unsigned)nq), dim3(kGroupThreads), 0, s, D, (int)nq, nprobe,
                     max_nprobe, k, Q, (uint32_t)item_budget,
                     (uint32_t)(scan_grid(D, item_budget) / (int)kXcds * scan_waves(D)), S);
}

void launch_scan(const Dev &D, int64_t nq, int nprobe, int max_nprobe, const float *Q, int item_budget,
                 const SearchScratch &S, hipStream_t s) {
  if (nq <= 0) return;
  if (D.pq_m > 0) {
    // parts per query, from the request's budget of work items: 32 items' worth to a workgroup
    int parts = (int)(item_budget / (nq * 32));
    parts = parts < 1 ? 1 : (parts > 64 ? 64 : parts);
    const size_t lds = (size_t)D.pq_m * 256 * sizeof(float);
    if (lds > 48 * 1024)  // with the kernel's own 8 KiB this passes the default limit of a workgroup
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_pq_scan),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(k_pq_scan, dim3((unsigned)(nq * parts)), dim3(kPqScanThreads), lds, s, D, nprobe,
                       max_nprobe, parts, S);
    return;
  }
  dim3 grid((unsigned)scan_grid(D, item_budget));
  const int waves = scan_waves(D);
  const size_t lds = (size_t)waves * kScanTileQueries * D.d * sizeof(float);
  const dim3 block(waves * kWave);
  switch (D.metric * 3 + D.storage) {
    case 0: hipLaunchKernelGGL((k_scan<0, 0>), grid, block, lds, s, D, max_nprobe, Q, S); break;
    case 1: hipLaunchKernelGGL((k_scan<0, 1>), grid, block, lds, s, D, max_nprobe, Q, S); break;
    case 2: hipLaunchKernelGGL((k_scan<0, 2>), grid, block, lds, s, D, max_nprobe, Q, S); break;
    case 3: hipLaunchKernelGGL((k_scan<1, 0>), grid, block, lds, s, D, max_nprobe, Q, S); break;
    case 4: hipLaunchKernelGGL((k_scan<1, 1>), grid, block, lds, s, D, max_nprobe, Q, S); break;
    default: hipLaunchKernelGGL((k_scan<1, 2>), grid, block, lds, s, D, max_nprobe, Q, S); break;
  }
}

void launch_select(const Dev &D, int64_t nq, int k, int nprobe, int max_nprobe,
                   const SearchScratch &S, float *out_dist, int64_t *out_ids, hipStream_t s) {
  if (nq <= 0) return;
  hipLaunchKernelGGL(k_select, dim3((unsigned)nq), dim3(kTopkThreads), 0, s, D, k, nprobe, max_nprobe,
                     S, out_dist, out_ids);
}

}  // namespace rtams
