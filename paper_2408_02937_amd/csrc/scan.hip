// The list scan of flat lists: exact scores of every query against every vector of its probed lists.
#include "search_common.h"

namespace rtams {

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
  uint32_t my_q = 0, my_len = 0, my_bound = 0;
  uint64_t my_keys = 0, my_poss = 0;  // addresses of the query's survivor records (keys, positions)
  if (lane < NQ) {
    const uint32_t pk = S.grouped[first + lane];
    my_q = pk >> 10;
    const size_t o = (size_t)my_q * max_nprobe + (pk & 1023u);
    my_len = S.probe_len[o];
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
          GlobalU32 *rk = (GlobalU32 *)(lane_u64(my_keys, i) + at);
          GlobalU32 *rp = (GlobalU32 *)(lane_u64(my_poss, i) + at);
          if ((m0[i] >> lane) & 1ull) {
            const uint32_t slot = (uint32_t)__popcll(m0[i] & below);
            rk[slot] = key_of_float((METRIC == 0 ? acc0[i] : -acc0[i]) + 0.0f);
            rp[slot] = slot_of(D, b0, (g0 % gpb) * kWave + (uint32_t)lane);
          }
          if ((m1[i] >> lane) & 1ull) {
            const uint32_t slot = (uint32_t)__popcll(m0[i]) + (uint32_t)__popcll(m1[i] & below);
            rk[slot] = key_of_float((METRIC == 0 ? acc1[i] : -acc1[i]) + 0.0f);
            rp[slot] = slot_of(D, b1, (g1 % gpb) * kWave + (uint32_t)lane);
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


void launch_scan(const Dev &D, int64_t nq, int nprobe, int max_nprobe, const float *Q, int item_budget,
                 const SearchScratch &S, hipStream_t s) {
  if (nq <= 0) return;
  if (D.pq_m > 0) {
    launch_pq_scan(D, nq, nprobe, max_nprobe, item_budget, S, s);
    return;
  }
  const ScanShape sh = scan_shape(D, item_budget);
  if (sh.mm) {
    launch_scan_mm(D, sh, max_nprobe, Q, S, s);
    return;
  }
  const dim3 grid((unsigned)sh.grid), block((unsigned)sh.threads);
  switch (D.metric * 3 + D.storage) {
    case 0: hipLaunchKernelGGL((k_scan<0, 0>), grid, block, sh.lds, s, D, max_nprobe, Q, S); break;
    case 1: hipLaunchKernelGGL((k_scan<0, 1>), grid, block, sh.lds, s, D, max_nprobe, Q, S); break;
    case 2: hipLaunchKernelGGL((k_scan<0, 2>), grid, block, sh.lds, s, D, max_nprobe, Q, S); break;
    case 3: hipLaunchKernelGGL((k_scan<1, 0>), grid, block, sh.lds, s, D, max_nprobe, Q, S); break;
    case 4: hipLaunchKernelGGL((k_scan<1, 1>), grid, block, sh.lds, s, D, max_nprobe, Q, S); break;
    default: hipLaunchKernelGGL((k_scan<1, 2>), grid, block, sh.lds, s, D, max_nprobe, Q, S); break;
  }
}

}  // namespace rtams
