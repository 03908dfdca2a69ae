// Top-k selection: the k best of every query's survivor records, by (score, id).
#include "search_common.h"

namespace rtams {

// ------------------------------------------------------------ top-k selection
// One workgroup per query takes the k best of the query's survivor records
// (what the scan appended for it) by (score, id): exact selection with the id
// tie-break, then a sort of the winners.  The records
// number a few hundred as a rule and are worked on in LDS; a list longer than
// LDS holds (massive ties) is selected from in place.
constexpr int kSurvivorCap = 4096;

constexpr int kTieCap = 1024;  // candidates tied at the k-th score that are told apart in LDS

struct SelectShared {
  __attribute__((aligned(8))) uint32_t hist[kSelectLdsWords];
  uint32_t bc[4];
  uint32_t cnt[2];
  uint64_t k1[kMaxK];
  uint64_t k2[kMaxK];
  uint32_t pay[kMaxK];
  uint64_t tie_id[kTieCap];
  uint32_t tie_item[kTieCap];
};

// Exact top-k among `count` items given by key(j) (32-bit score key) and
// item(j) (the candidate's place in the pool, for the id lookup).  Leaves the winners sorted in
// sh.k1 (score key), sh.k2 (id key), sh.pay (place in the pool); returns how
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
                                                        const float *__restrict__ Q, SearchScratch S,
                                                        float *__restrict__ out_dist,
                                                        int64_t *__restrict__ out_ids) {
  __shared__ SelectShared sh;
  __shared__ uint32_t skey[kSurvivorCap];
  __shared__ uint32_t sidx[kSurvivorCap];
  __shared__ uint32_t scount;
  const int q = blockIdx.x;
  const int n = (int)S.rec_cnt[q];
  const unsigned long long base = S.qbase[q];
  const uint32_t *rk = rec_keys_of(S, base), *rp = rec_poss_of(S, base);
  const int metric = D.metric;
  const int lane = threadIdx.x & (kWave - 1);
  if (threadIdx.x == 0) scount = 0;
  __syncthreads();

  // The records are taken into LDS in portions.  Once LDS is more than half full the k-th best
  // of what it holds becomes the limit (it cannot be better than the final k-th best): what is
  // worse is dropped, and later portions are filtered on the way in.  Under a limit only a few
  // per cent of a portion pass as a rule, so a portion is four times what LDS could take if all
  // of it passed; should it not fit after all, what it added is dropped, the limit is renewed
  // and the portion is read again, cut to what fits for certain.  Ties that no limit can
  // separate (LDS stays more than half full) are left to the selection in place below.
  // With norm-form scores among the records (flat float lists under L2 scored on the matrix cores) a
  // limit taken from the k-th best record is loosened twice: once to bound the k-th best direct-form
  // score from above, once more to admit every record whose direct-form score may reach that.
  const bool approx = uses_norm_form(D);
  const float slack = norm_form_slack(D.d), qn = approx ? S.qnorm[q] : 0.f;
  auto limit_from = [&](uint32_t kth) {
    return approx ? loosened_key(loosened_key(kth, slack, qn), slack, qn) : kth;
  };
  // what LDS holds is cut down to the records not worse than the limit: everybody reads its
  // entries, then everybody writes the kept ones back
  auto keep_not_worse = [&](int have, uint32_t lim) {
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
      const bool keep = j < have && mk[u] <= lim;
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
  };
  uint32_t limit = S.bound[q];
  bool in_lds = true;
  __shared__ uint32_t s_over;
  int stretch = 1;  // portions as a multiple of the room in LDS
  // More records than LDS holds (the query's bound was loose: its sample did not look like its
  // candidates): a first limit comes from a pilot, every (n / pilot)-th record, so that the
  // records are filtered from the first portion on instead of filling LDS once unfiltered.  A query
  // with tens of thousands of records (a hot list) takes a pilot as large as LDS: the k-th best of
  // 4096 lets about k / 4096 of the records pass, which fit in one go.
  constexpr int kPilot = 1024;
  if (n > kSurvivorCap && k <= kPilot) {  // uniform over the workgroup
    const int pilot = n >= 8 * kSurvivorCap ? kSurvivorCap : kPilot;
    const int stride = n / pilot;
    for (int j = threadIdx.x; j < pilot; j += kTopkThreads) skey[j] = rk[(size_t)j * stride];
    __syncthreads();
    const SelectResult r = wg_radix_select<32>(
        pilot, (uint32_t)k, [&](int j, uint64_t &kv) { kv = skey[j]; return true; }, sh.hist, sh.bc);
    const uint32_t lim = limit_from((uint32_t)r.T);
    limit = lim < limit ? lim : limit;
    stretch = pilot == kSurvivorCap ? 16 : 4;
    __syncthreads();  // the pilot's keys are done with
  }
  // A query whose records take several round trips to stream keeps, of a record that passes, its
  // index first and fetches the positions of what LDS holds in the end (the positions of the many
  // that do not pass are never read); a query that is through in one round trip loads both together.
  // 16 keys in flight per thread either way (24 or 32 take the kernel past 128 registers).
  const bool deferred = n > 16 * kTopkThreads;  // uniform over the workgroup
  auto stream = [&](auto tag, int next, int m) {
    constexpr bool kDeferred = decltype(tag)::value;
    constexpr int kInFlight = kDeferred ? 16 : 16;
    for (int j0 = 0; j0 < m; j0 += kInFlight * kTopkThreads) {
      uint32_t kv[kInFlight], pv[kDeferred ? 1 : kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {  // clamped index: the loads are unconditional and issue back to back
        const int j = j0 + u * kTopkThreads + (int)threadIdx.x;
        kv[u] = rk[next + (j < m ? j : m - 1)];
      }
      if (!kDeferred) {
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
          const int j = j0 + u * kTopkThreads + (int)threadIdx.x;
          pv[u] = rp[next + (j < m ? j : m - 1)];
        }
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
            if (slot < (uint32_t)kSurvivorCap) { skey[slot] = kv[u]; sidx[slot] = kDeferred ? (uint32_t)(next + j) : pv[kDeferred ? 0 : u]; }
            else s_over = 1u;
          }
        }
      }
    }
  };
  for (int next = 0; next < n;) {  // every branch here is uniform over the workgroup
    const int count = (int)scount;
    const int m = min(n - next, stretch * (kSurvivorCap - count));
    if (threadIdx.x == 0) s_over = 0;
    __syncthreads();
    // (the positions come with the keys, or afterwards, but never from inside the filter loop: a load
    // there, for the records that pass, would make every turn of it a round trip of its own)
    if (deferred) stream(std::true_type{}, next, m);
    else stream(std::false_type{}, next, m);
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
      const uint32_t lim = limit_from((uint32_t)r.T);
      limit = lim < limit ? lim : limit;
      keep_not_worse(have, limit);  // drop what is worse
      if ((int)scount > kSurvivorCap / 2) { in_lds = false; break; }
    }
    // from the first limit on, portions may be stretched; a portion that did not fit is read
    // again unstretched (it fits then, whatever it holds)
    stretch = over ? 1 : 4;
  }

  if (deferred && in_lds) {  // uniform: LDS holds indices of records; now their places in the pool
    __syncthreads();
    const int have = (int)scount;
    for (int j = threadIdx.x; j < have; j += kTopkThreads) sidx[j] = rp[sidx[j]];
    __syncthreads();
  }
  // a record's place in the pool (slot_of) -> which block, which place in it
  auto locate = [&](int i, uint32_t &b, uint32_t &moff) {
    b = (uint32_t)i / (uint32_t)D.T_m;
    moff = (uint32_t)i - b * (uint32_t)D.T_m;
  };
  auto id_of = [&](int i) -> int64_t {
    uint32_t b, moff;
    locate(i, b, moff);
    return block_ids(D, b)[moff];
  };
  // place in the pool -> key of the candidate's direct-form squared distance.  Four neighbouring lanes share
  // a candidate (a vector's chunks of 4 dimensions lie 1 KiB apart: every chunk is a memory
  // transaction of its own, and this way all of them are in flight at once): lane s of the four
  // takes chunks s, s + 4, ..., and the four partial sums are added pairwise.  All four lanes call
  // this with the same place and get the key.
  auto direct_key = [&](int i, int64_t *id) -> uint32_t {
    uint32_t b, moff;
    locate(i, b, moff);
    const int sub = (int)(threadIdx.x & 3u);
    if (id && sub == 0) *id = block_ids(D, b)[moff];
    const float4 *__restrict__ x =
        block_vecs(D, b) + (size_t)(moff / kWave) * D.d4 * kWave + (moff & (kWave - 1));
    const float4 *__restrict__ y = reinterpret_cast<const float4 *>(Q + (size_t)q * D.d);
    float acc = 0.f;
    int c = sub;
    for (; c + 28 < D.d4; c += 32) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = x[(size_t)(c + 4 * u) * kWave];
#pragma unroll
      for (int u = 0; u < 8; ++u) accumulate<0>(acc, v[u], y[c + 4 * u]);
    }
    for (; c < D.d4; c += 4) accumulate<0>(acc, x[(size_t)c * kWave], y[c]);
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    return key_of_float(acc + 0.0f);
  };
  // The same for two candidates at once: both block look-ups go out together, then all the chunks of
  // both (a candidate is a chain of two round trips to memory; two of them side by side cost one).
  auto direct_key_pair = [&](int ia, int ib, int64_t *ida, int64_t *idb, uint32_t &ka, uint32_t &kb) {
    uint32_t ba, ma, bb, mb;
    locate(ia, ba, ma);
    locate(ib, bb, mb);
    const int sub = (int)(threadIdx.x & 3u);
    if (sub == 0) {
      *ida = block_ids(D, ba)[ma];
      *idb = block_ids(D, bb)[mb];
    }
    const float4 *__restrict__ xa = block_vecs(D, ba) + (size_t)(ma / kWave) * D.d4 * kWave + (ma & (kWave - 1));
    const float4 *__restrict__ xb = block_vecs(D, bb) + (size_t)(mb / kWave) * D.d4 * kWave + (mb & (kWave - 1));
    const float4 *__restrict__ y = reinterpret_cast<const float4 *>(Q + (size_t)q * D.d);
    float acca = 0.f, accb = 0.f;
    int c = sub;
    for (; c + 28 < D.d4; c += 32) {
      float4 va[8], vb[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) va[u] = xa[(size_t)(c + 4 * u) * kWave];
#pragma unroll
      for (int u = 0; u < 8; ++u) vb[u] = xb[(size_t)(c + 4 * u) * kWave];
#pragma unroll
      for (int u = 0; u < 8; ++u) accumulate<0>(acca, va[u], y[c + 4 * u]);
#pragma unroll
      for (int u = 0; u < 8; ++u) accumulate<0>(accb, vb[u], y[c + 4 * u]);
    }
    for (; c < D.d4; c += 4) {
      const float4 va = xa[(size_t)c * kWave], vb = xb[(size_t)c * kWave];
      accumulate<0>(acca, va, y[c]);
      accumulate<0>(accb, vb, y[c]);
    }
    acca += __shfl_xor(acca, 1);
    acca += __shfl_xor(acca, 2);
    accb += __shfl_xor(accb, 1);
    accb += __shfl_xor(accb, 2);
    ka = key_of_float(acca + 0.0f);
    kb = key_of_float(accb + 0.0f);
  };
  int kk = -1;
  if (approx && in_lds) {  // uniform over the workgroup
    // The usual case: the finalists (every record that may be among the k best by direct-form
    // scores, i.e. not worse than the twice loosened k-th best of what LDS holds) number little
    // more than k.  They get their direct-form scores and ids in one go and are sorted by those.
    const int have = (int)scount;
    uint32_t lim = 0xFFFFFFFFu;
    if (have > k) {
      const SelectResult r = wg_radix_select<32>(
          have, (uint32_t)k, [&](int j, uint64_t &kv) { kv = skey[j]; return true; }, sh.hist, sh.bc);
      lim = limit_from((uint32_t)r.T);
      limit = lim < limit ? lim : limit;
    }
    if (threadIdx.x == 0) sh.cnt[0] = 0;
    __syncthreads();
    for (int j = threadIdx.x; j < have; j += kTopkThreads)
      if (skey[j] <= lim) {
        const uint32_t p = atomicAdd(&sh.cnt[0], 1u);
        if (p < (uint32_t)kMaxK) sh.pay[p] = sidx[j];
      }
    __syncthreads();
    const int m = (int)sh.cnt[0];
    if (m <= kMaxK) {
      constexpr int kFours = kTopkThreads / 4;
      for (int p0 = 0; p0 < m;) {  // uniform trip count: the lanes of a four stay together
        const int p = p0 + (int)(threadIdx.x >> 2);
        if (m - p0 > kFours) {  // uniform: every four takes two finalists, p and p + kFours
          const int p2 = p + kFours;
          int64_t id = 0, id2 = 0;
          uint32_t key, key2;
          direct_key_pair((int)sh.pay[p < m ? p : m - 1], (int)sh.pay[p2 < m ? p2 : m - 1], &id, &id2, key, key2);
          if ((threadIdx.x & 3u) == 0) {
            if (p < m) { sh.k1[p] = key; sh.k2[p] = (uint64_t)id ^ 0x8000000000000000ull; }
            if (p2 < m) { sh.k1[p2] = key2; sh.k2[p2] = (uint64_t)id2 ^ 0x8000000000000000ull; }
          }
          p0 += 2 * kFours;
        } else {
          int64_t id = 0;
          const uint32_t key = direct_key((int)sh.pay[p < m ? p : m - 1], &id);
          if (p < m && (threadIdx.x & 3u) == 0) {
            sh.k1[p] = key;
            sh.k2[p] = (uint64_t)id ^ 0x8000000000000000ull;
          }
          p0 += kFours;
        }
      }
      wg_sort(m, sh.k1, sh.k2, sh.pay);
      kk = k < m ? k : m;
    }
  }
  if (approx && kk < 0) {  // uniform over the workgroup
    // Many finalists (near-ties by the thousand): whatever is not worse than the limit is scored
    // again where it lies, and the selection then runs on direct-form scores as for the other kinds of list.
    if (in_lds) {
      keep_not_worse((int)scount, limit);
      const int have = (int)scount;
      for (int j0 = 0; j0 < have; j0 += kTopkThreads / 4) {
        const int j = j0 + (int)(threadIdx.x >> 2);
        const uint32_t key = direct_key((int)sidx[j < have ? j : have - 1], nullptr);
        if (j < have && (threadIdx.x & 3u) == 0) skey[j] = key;
      }
    } else {
      // the records are this query's own
      uint32_t *wk = const_cast<uint32_t *>(rk);
      for (int j0 = 0; j0 < n; j0 += kTopkThreads / 4) {
        const int j = j0 + (int)(threadIdx.x >> 2);
        const int jj = j < n ? j : n - 1;
        const bool want = rk[jj] <= limit;
        uint32_t key = 0xFFFFFFFFu;
        if (__any(want)) {  // uniform over the wavefront, so the fours stay together
          const uint32_t dk = direct_key((int)rp[jj], nullptr);
          key = want ? dk : key;
        }
        if (j < n && (threadIdx.x & 3u) == 0) wk[j] = key;
      }
    }
    __syncthreads();
  }
  if (kk < 0) {
    if (in_lds)
      kk = select_topk((int)scount, k, [&](int j) { return skey[j]; }, [&](int j) { return (int)sidx[j]; },
                       id_of, sh);
    else
      kk = select_topk(n, k, [&](int j) { return rk[j]; }, [&](int j) { return (int)rp[j]; }, id_of, sh);
  }

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


void launch_select(const Dev &D, int64_t nq, int k, int nprobe, int max_nprobe, const float *Q,
                   const SearchScratch &S, float *out_dist, int64_t *out_ids, hipStream_t s) {
  if (nq <= 0) return;
  hipLaunchKernelGGL(k_select, dim3((unsigned)nq), dim3(kTopkThreads), 0, s, D, k, nprobe, max_nprobe,
                     Q, S, out_dist, out_ids);
}

}  // namespace rtams
