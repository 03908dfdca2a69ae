// Probe selection and the per-query plan of a search request.
// (Paper, introduction: a query is compared with the lists of the clusters nearest to it only.)
#include "search_common.h"

namespace rtams {

// Workgroup of the probe selection: 256 threads, or 1024 where a query has thousands of centroids to
// go through (every pass of the selection reads them all).
constexpr int kSelThreads = 256, kSelThreadsMany = 1024, kSelManyFrom = 4096;

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
__global__ __launch_bounds__(kSelThreadsMany) void k_probe_plan(Dev D, int nprobe, int max_nprobe,
                                                            SearchScratch S, const float *__restrict__ Q,
                                                            int32_t *probe_out) {
  __shared__ __attribute__((aligned(8))) uint32_t hist[kSelectLdsWords];
  __shared__ uint32_t bc[4];
  __shared__ uint32_t cnt[2];
  __shared__ uint64_t k1[kMaxNprobe];
  __shared__ uint64_t k2[kMaxNprobe];
  __shared__ uint32_t pay[kMaxNprobe];
  __shared__ float s_red[kSelThreadsMany / kWave];
  const int T = (int)blockDim.x;
  const int q = blockIdx.x;
  const int n = D.nlist;
  double *sc = S.scores + (size_t)q * n;
  const int metric = D.metric;
  // the fixed arithmetic of coarse.hip for one centroid: a chain of multiply-adds in the order of the
  // coordinates, fed by 16-byte loads that run eight chunks ahead of it (one coordinate per load, each
  // waited for, made a candidate of 768 dimensions cost a hundred nanoseconds per coordinate)
  auto exact = [&](int c) -> double {
    const float4 *y4 = reinterpret_cast<const float4 *>(Q + (size_t)q * D.d);
    const float4 *r4 = reinterpret_cast<const float4 *>(D.centroids + (size_t)c * D.d);
    const int d4 = D.d4;
    double acc = 0.0;
    auto chain = [&](const float4 &y, const float4 &r) {
      if (metric == 0) {
        const double t0 = (double)y.x - (double)r.x; acc = __builtin_fma(t0, t0, acc);
        const double t1 = (double)y.y - (double)r.y; acc = __builtin_fma(t1, t1, acc);
        const double t2 = (double)y.z - (double)r.z; acc = __builtin_fma(t2, t2, acc);
        const double t3 = (double)y.w - (double)r.w; acc = __builtin_fma(t3, t3, acc);
      } else {
        acc = __builtin_fma((double)y.x, (double)r.x, acc);
        acc = __builtin_fma((double)y.y, (double)r.y, acc);
        acc = __builtin_fma((double)y.z, (double)r.z, acc);
        acc = __builtin_fma((double)y.w, (double)r.w, acc);
      }
    };
    int j = 0;
    for (; j + 8 <= d4; j += 8) {
      float4 a[8], b[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) { a[u] = y4[j + u]; b[u] = r4[j + u]; }
#pragma unroll
      for (int u = 0; u < 8; ++u) chain(a[u], b[u]);
    }
    for (; j < d4; ++j) chain(y4[j], r4[j]);
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
    for (int j = threadIdx.x; j < D.d; j += T) { const float v = Q[(size_t)q * D.d + j]; yn = fmaf(v, v, yn); }
    for (int o = kWave / 2; o > 0; o >>= 1) yn += __shfl_xor(yn, o);
    if ((threadIdx.x & (kWave - 1)) == 0) s_red[threadIdx.x / kWave] = yn;
    __syncthreads();
    yn = 0.f;
    for (int w = 0; w < T / kWave; ++w) yn += s_red[w];
    const float cmax = __uint_as_float(D.ctrl->cnorm_max_bits);
    const float band = coarse_band(D.d, yn + cmax) * 1.01f;  // 2 E, see coarse_mfma.hip
    const SelectResult ra = wg_radix_select<32>(
        n, (uint32_t)nprobe, [&](int i, uint64_t &k) { k = key_of_float(ap[i] + 0.0f); return true; }, hist, bc);
    const uint32_t tk = (uint32_t)ra.T;  // key of (an upper bound of) the nprobe-th smallest approximation
    const float t = __uint_as_float((tk & 0x80000000u) ? (tk & 0x7fffffffu) : ~tk);
    const float limit = t + band;
    if (threadIdx.x == 0) cnt[0] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += T)
      if (ap[i] <= limit) {
        uint32_t p = atomicAdd(&cnt[0], 1u);
        if (p < (uint32_t)kMaxNprobe) pay[p] = (uint32_t)i;
      }
    __syncthreads();
    const int nc = (int)cnt[0];
    if (nc >= nprobe && nc <= kMaxNprobe) {  // (fewer than nprobe: scores that do not compare, e.g. NaN)
      for (int p = threadIdx.x; p < nc; p += T) {
        const int c = (int)pay[p];
        k1[p] = key_of_score(exact(c));
        k2[p] = (uint64_t)c;
      }
      wg_sort(nc, k1, k2, pay);  // by (exact score, index): the first nprobe are the answer
      done = true;
    } else {
      for (int i = threadIdx.x; i < n; i += T) sc[i] = exact(i);  // the filter did not narrow it: whole row
      __syncthreads();
    }
  }
  auto key1 = [&](int i) -> uint64_t { return key_of_score(sc[i]); };

  SelectResult r1{~0ull, 0, 0}, r2{~0ull, 0, 0};
  const bool all = nprobe >= n;
  if (!done && FROM_APPROX && all) {  // every list is probed: exact order of the whole row
    for (int i = threadIdx.x; i < n; i += T) sc[i] = exact(i);
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
  for (int i = threadIdx.x; i < n; i += T) {
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
    for (int p = threadIdx.x; p < nprobe; p += T) pay[p] = (uint32_t)k2[p];
    __syncthreads();
  }

  // plan
  int32_t *pl = S.probe_list + (size_t)q * max_nprobe;
  uint32_t *plen = S.probe_len + (size_t)q * max_nprobe;
  for (int p = threadIdx.x; p < nprobe; p += T) {
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
      tot += pay[p];
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
      for (int p = 0; p < nprobe; ++p) plen[p] = 0;
    }
    S.qbase[q] = base;
    S.qtotal[q] = (uint32_t)tot;
  }
}


void launch_probe_plan(const Dev &D, int64_t nq, int nprobe, int max_nprobe, const SearchScratch &S,
                       const float *Q, bool from_approx, int32_t *probe_out, hipStream_t s) {
  if (nq <= 0) return;
  const unsigned threads = D.nlist >= kSelManyFrom ? kSelThreadsMany : kSelThreads;
  if (from_approx)
    hipLaunchKernelGGL(k_probe_plan<true>, dim3((unsigned)nq), dim3(threads), 0, s, D, nprobe, max_nprobe,
                       S, Q, probe_out);
  else
    hipLaunchKernelGGL(k_probe_plan<false>, dim3((unsigned)nq), dim3(threads), 0, s, D, nprobe, max_nprobe,
                       S, Q, probe_out);
}

}  // namespace rtams
