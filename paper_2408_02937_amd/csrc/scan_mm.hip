// The list scan of flat float lists on the matrix cores.
#include "search_common.h"

namespace rtams {

// The scores of a tile are a small dense contraction (vectors x queries over the dimensions), and the
// interleaved layout hands a wavefront exactly the operand the 4x4x1 matrix instruction wants: lane =
// vector, one coordinate per instruction (search_common.h).  A workgroup takes one work item (list,
// segment, tile of up to 32 of the queries probing the list).  The tile's queries go to LDS once, in
// groups of four (rows past the tile's last query are zero), each with the words the scan needs of
// it: how far its list goes, its bound, where its survivor records go.  Then the four wavefronts share
// out the segment's groups of 64 vectors and work on their own: per chunk of 4 dimensions a wavefront
// loads 1 KiB ONCE, lane l reads the float4 of query 4 g + l % 4 of every group of queries g, and four
// matrix instructions per group of queries use them up.  Per 1 KiB of list data that is 4 matrix
// instructions of 8 cycles for every 4 queries, against 16 to 32 vector instructions of 4 cycles, and
// the vector unit is left with |x|^2 (squared distances only): the kernel sits on the memory side,
// and a list is read once per 32 of the queries that probe it.
// Inner products are returned as the contraction leaves them (the bound's sample uses the same
// instruction sequence, so a pair scores the same bits there and here).  Squared distances take the
// norm form |x|^2 + |q|^2 - 2 <x, q>, whose rounding errors scale with the norms: the bound they are
// compared with was loosened by the proven margin, and the selection scores its finalists again in
// the direct form, so what is returned is exactly what the direct form gives.
// Afterwards lane l holds, for each group of queries g, the scores of vectors 4 (l / 4) .. + 3 against
// ONE query, 4 g + l % 4.  What is not worse than that query's bound goes to a staging area of the
// wavefront in LDS (places from ballots, no waiting); when the area is full, and when the wavefront
// is through with its groups, the staged survivors are counted per query with LDS atomics, ONE
// global atomic instruction reserves the places of all the tile's queries, and the records go out.
// (A returning global atomic per group of queries and of vectors, waited for each time, cost more
// than the scan itself: dozens of wavefronts reserve from the same few counters.)

struct TileQuery {  // kMmQueryWords 32-bit words
  uint32_t q, len, bound;
  float qn;
  uint32_t pad[4];
  uint64_t keys, poss;  // addresses of the query's survivor records (keys, positions)
};
static_assert(sizeof(TileQuery) == kMmQueryWords * 4, "words per query of a tile");

struct WaveStage {  // survivors of one wavefront on their way out
  uint32_t key[kMmStageCap], pos[kMmStageCap];
  uint8_t row[kMmStageCap];  // which query of the tile
  uint32_t qcnt[kMmTileMax], qbase[kMmTileMax];
};
static_assert(sizeof(WaveStage) == kMmStageBytes, "staging bytes per wavefront");

// The groups g_lo + wave, g_lo + wave + 4, ... below g_hi of the list against QG groups of four queries.
// first_b: the block that holds the wavefront's first group (looked up by the caller).
template <int METRIC, int QG>
__device__ __forceinline__ void scan_groups_mm(const Dev &D, const SearchScratch &S, int list, uint32_t g_lo,
                                               uint32_t g_hi, uint32_t first_b, const float4 *qs,
                                               const TileQuery *tq, WaveStage &st) {
  constexpr int kPrefetch = 4;  // chunks per register set: 8 KiB of loads in flight per wavefront
  const int d4 = D.d4;
  const int qstride = d4 + 1;  // float4s between two queries in LDS: an odd stride keeps the four rows a read touches on different banks
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane & 3;
  const float4 *__restrict__ qrow = qs + sub * qstride;  // query `sub` of group 0; group g is 4 g rows on
  const uint32_t gpb = (uint32_t)D.groups_per_block;
  const size_t group_stride = (size_t)d4 * kWave;
  uint32_t staged = 0;  // survivors in the staging area (uniform over the wavefront)
  auto wave_sync = [] {  // LDS operations of one wavefront execute in order; keep the compiler from moving them
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };
  auto flush = [&]() __attribute__((always_inline)) {
    if (lane < kMmTileMax) st.qcnt[lane] = 0u;
    wave_sync();
    constexpr int kMine = kMmStageCap / kWave;
    uint32_t rank[kMine], row[kMine];
#pragma unroll
    for (int u = 0; u < kMine; ++u) {
      const uint32_t e = (uint32_t)lane + u * kWave;
      row[u] = e < staged ? st.row[e] : 0u;
      rank[u] = e < staged ? atomicAdd(&st.qcnt[row[u]], 1u) : 0u;  // place among the query's survivors of this flush
    }
    wave_sync();
    if (lane < kMmTileMax) {
      const uint32_t c = st.qcnt[lane];
      st.qbase[lane] = c ? atomicAdd(&S.rec_cnt[tq[lane].q], c) : 0u;  // rows past the tile's last query have none
    }
    wave_sync();
#pragma unroll
    for (int u = 0; u < kMine; ++u) {
      const uint32_t e = (uint32_t)lane + u * kWave;
      if (e < staged) {
        // (a pointer rebuilt from integers has no address space: say "global", or the stores become FLAT
        // operations, and while one of those is pending every wait of the load pipeline has to be for
        // ALL outstanding memory operations)
        const uint64_t at = 4ull * (st.qbase[row[u]] + rank[u]);
        *(GlobalU32 *)(tq[row[u]].keys + at) = st.key[e];
        *(GlobalU32 *)(tq[row[u]].poss + at) = st.pos[e];
      }
    }
    wave_sync();
    staged = 0;
  };
  // The wavefront's groups of vectors as a software pipeline ACROSS the groups: while one is being
  // streamed the block number of the next is looked up, and the first loads of the next go out before
  // the survivors of this one are dealt with, so that neither the two dependent table reads nor the
  // first trip to memory of a group stand between two groups (a quarter of a group's time at d = 128).
  const int d4_main = d4 & ~(2 * kPrefetch - 1);  // chunks that go through the two register sets
  float4 sa[kPrefetch], sb[kPrefetch];
  auto load_set = [&](float4 *s, const float4 *__restrict__ p, int cb) {
#pragma unroll
    for (int u = 0; u < kPrefetch; ++u) s[u] = p[(size_t)(cb + u) * kWave];
    __builtin_amdgcn_sched_barrier(0);  // loads are issued here, not sunk towards their use
  };
  auto place = [&](uint32_t g, uint32_t b) -> const float4 * {
    return block_vecs(D, b) + (size_t)(g % gpb) * group_stride + lane;
  };
  uint32_t g0 = g_lo + (uint32_t)wave;
  if (g0 >= g_hi) return;  // nothing staged yet
  const float4 *x = place(g0, first_b);
  uint32_t cur_b = first_b;  // the block of group g0
  if (d4_main) load_set(sa, x, 0);
  for (;;) {
    const uint32_t g_next = g0 + kMmWaves;
    const bool more = g_next < g_hi;  // uniform over the wavefront
    uint32_t next_b = 0;
    if (more) next_b = (uint32_t)*table_entry(D, list, g_next / gpb);  // on its way while this group is streamed
    MfmaAcc acc[QG];
#pragma unroll
    for (int g = 0; g < QG; ++g) acc[g] = (MfmaAcc){0.f, 0.f, 0.f, 0.f};
    float nrm = 0.f;  // |x|^2 of the lane's own vector
    // every accumulator takes the coordinates in their order; the chains of the groups of queries are
    // interleaved so that no instruction waits for the one in front of it
    auto use = [&](const float4 &v, int c) {
      if (METRIC == 0) accumulate<1>(nrm, v, v);
      constexpr int kHalf = QG == 6 ? 3 : QG > 4 ? 4 : QG;  // groups of queries whose coordinates are held at once (a divisor of QG)
#pragma unroll
      for (int h = 0; h < QG; h += kHalf) {
        float4 y[kHalf];
#pragma unroll
        for (int g = 0; g < kHalf; ++g) y[g] = qrow[4 * (h + g) * qstride + c];
#pragma unroll
        for (int g = 0; g < kHalf; ++g) mfma_step(acc[h + g], v.x, y[g].x);
#pragma unroll
        for (int g = 0; g < kHalf; ++g) mfma_step(acc[h + g], v.y, y[g].y);
#pragma unroll
        for (int g = 0; g < kHalf; ++g) mfma_step(acc[h + g], v.z, y[g].z);
#pragma unroll
        for (int g = 0; g < kHalf; ++g) mfma_step(acc[h + g], v.w, y[g].w);
      }
    };
    auto use_set = [&](const float4 *s, int cb) {
#pragma unroll
      for (int u = 0; u < kPrefetch; ++u) use(s[u], cb + u);
      __builtin_amdgcn_sched_barrier(0);
    };
    if (d4_main) {  // set a holds chunks 0 .. kPrefetch - 1 of this group already
      int c = 0;
#pragma unroll 1
      for (; c + 2 * kPrefetch < d4_main; c += 2 * kPrefetch) {
        load_set(sb, x, c + kPrefetch);
        use_set(sa, c);
        load_set(sa, x, c + 2 * kPrefetch);
        use_set(sb, c + kPrefetch);
      }
      load_set(sb, x, c + kPrefetch);
      use_set(sa, c);
      use_set(sb, c + kPrefetch);
    }
    for (int c = d4_main; c < d4; ++c) use(x[(size_t)c * kWave], c);
    const float4 *x_next = x;
    if (more) {  // the next group's first loads go out before this group's survivors are dealt with
      x_next = place(g_next, next_b);
      if (d4_main) load_set(sa, x_next, 0);
    }

    // scores -> keys; which of the lane's 4 candidates per group of queries survive
    const float nr[4] = {quad_broadcast<0>(nrm), quad_broadcast<1>(nrm), quad_broadcast<2>(nrm), quad_broadcast<3>(nrm)};
    const uint32_t vbase = g0 * kWave + 4u * (uint32_t)(lane >> 2);
    const uint32_t slot_base = slot_of(D, cur_b, (g0 % gpb) * kWave + 4u * (uint32_t)(lane >> 2));
#pragma unroll
    for (int g = 0; g < QG; ++g) {
      const TileQuery me = tq[4 * g + sub];  // len 0 for rows past the tile: nothing of theirs is kept
      uint32_t key[4], pass = 0u;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float sc = acc[g][r];
        sc = METRIC == 0 ? fmaf(-2.f, sc, nr[r] + me.qn) : -sc;
        key[r] = key_of_float(sc + 0.0f);
        if (vbase + r < me.len && key[r] <= me.bound) pass |= 1u << r;
      }
      if (__ballot(pass != 0u) == 0ull) continue;  // uniform
      // places in the staging area: candidate r of every lane, lane after lane, then candidate r + 1
      uint32_t at[4], total = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const unsigned long long m = __ballot((pass >> r) & 1u);
        at[r] = total + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        total += (uint32_t)__popcll(m);
      }
      if (staged + total > (uint32_t)kMmStageCap) flush();  // uniform; at most 4 x 64 at once: they always fit an empty area
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (pass & (1u << r)) {
          const uint32_t e = staged + at[r];
          st.key[e] = key[r];
          st.pos[e] = slot_base + r;
          st.row[e] = (uint8_t)(4 * g + sub);
        }
      staged += total;
    }
    if (!more) break;
    g0 = g_next;
    x = x_next;
    cur_b = next_b;
  }
  if (staged) flush();
}

// Hardware hands consecutive workgroup ids to the 8 XCDs in turn, so workgroup i runs on XCD i % 8 and
// takes item i / 8 of that XCD's range of items (a contiguous range of lists); workgroups past the end
// of their range leave at once.
// STEAL (long scans): the ranges are cut for equal cost, but the XCDs do not finish together (measured
// at 20 M x 256: the last one 5 to 14 % behind the average), so a workgroup whose XCD has no item left
// for it takes one from the BACK of another XCD's range.  All such workgroups of an XCD go to the same
// victim first (the next XCD that is not done) and get neighbouring items: the tiles of one segment,
// which then come from memory once for this XCD too.  Whoever takes an item, owner or not, takes it
// by swapping the descriptor's pair count for zero, so every item is scanned exactly once; an owner
// that finds its item gone goes looking as well.  A victim whose back has met its front (a swap that
// found zero, or no item left) is marked done and not asked again.  Nobody waits for anybody: a
// workgroup that finds nothing leaves.  Short scans keep the plain mapping: the swap is a round trip
// in front of every item, and the launch has tens of thousands of workgroups that find their range
// used up and should leave at once (measured at 1 M x 128, 2,048 items: 226 instead of 103 us).
template <int METRIC, bool STEAL>
__global__ __launch_bounds__(kMmWaves *kWave) void k_scan_mm(Dev D, int max_nprobe, const float *__restrict__ Q,
                                                             SearchScratch S, int tile_rows) {
  extern __shared__ float4 lds_mm[];  // [tile_rows][d / 4 + 1] coordinates of the tile's queries, [tile_rows] TileQuery, [wavefronts] WaveStage
  ScanQueues *Qs = S.queues;
  const uint32_t xcd = blockIdx.x % kXcds;
  const uint32_t own = Qs->begin[xcd] + blockIdx.x / kXcds;
  const bool has_own = own < Qs->begin[xcd + 1];
  if (!STEAL && !has_own) return;
  const uint32_t seg = Qs->seg_groups;
  if (seg == 0) return;
  uint4 desc = has_own ? S.tile_desc[own] : make_uint4(0u, 0u, 0u, 0u);  // (STEAL: on its way while thread 0 takes the item)
  uint32_t pairs = desc.z;
  if (STEAL) {
    __shared__ uint32_t s_item, s_pairs;
    if (threadIdx.x == 0) {
      uint32_t item = own, got = 0u;
      if (has_own) got = atomicExch(&S.tile_desc[own].z, 0u);
      if (!got) {
        const uint32_t all = (1u << kXcds) - 1u;
        uint32_t done = __hip_atomic_load(&Qs->done_mask, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) | (1u << xcd);
        for (uint32_t k = 1; k < kXcds && !got && done != all; ++k) {
          const uint32_t y = (xcd + k) % kXcds;
          if ((done >> y) & 1u) continue;
          const uint32_t count = Qs->begin[y + 1] - Qs->begin[y];
          const uint32_t b = atomicAdd(&Qs->back[y], 1u);
          if (b < count) {
            item = Qs->begin[y + 1] - 1u - b;
            got = atomicExch(&S.tile_desc[item].z, 0u);
          }
          if (!got) {
            atomicOr(&Qs->done_mask, 1u << y);
            done |= 1u << y;
          }
        }
      }
      s_item = item;
      s_pairs = got;
    }
    __syncthreads();
    pairs = s_pairs;
    if (pairs == 0) return;  // uniform over the workgroup
    // (a workgroup without an item of its own computed an `own` beyond its range, which may be the very
    // number of the item it took from the next XCD: what it loaded above was nothing)
    if (!has_own || s_item != own) desc = S.tile_desc[s_item];
  }
  const int list = (int)desc.x;
  const uint32_t first = desc.y;
  if (pairs == 0) return;
  const int d4 = D.d4, qstride = d4 + 1;
  float4 *qs = lds_mm;
  TileQuery *tq = reinterpret_cast<TileQuery *>(lds_mm + (size_t)tile_rows * qstride);
  WaveStage &st = reinterpret_cast<WaveStage *>(tq + tile_rows)[threadIdx.x / kWave];
  // groups of four queries of this tile: 1, 2, 3, 4, 6 or 8, whichever holds the item's queries; exactly
  // that many rows of LDS are set up, and the instantiation below reads exactly that many (the plan never
  // puts more queries into a tile than tile_rows)
  int qg = (int)((pairs + 3u) / 4u);
  qg = qg == 5 ? 6 : qg == 7 ? 8 : qg;
  const int rows = 4 * qg;
  if (rows > tile_rows || rows > kMmTileMax) return;  // a descriptor the launch was not sized for: nothing is scanned
  // The block number of the wavefront's first group of vectors is asked for now (two dependent reads)
  // and used after the tile is set up.  Never past the list's chain, whatever the descriptors say.
  const uint32_t g_begin = desc.w * seg;
  const uint32_t g_have = D.nblk[list] * (uint32_t)D.groups_per_block;
  uint32_t first_b = 0;
  {
    const uint32_t g0 = g_begin + threadIdx.x / kWave;
    if (g0 < g_have) first_b = (uint32_t)*table_entry(D, list, g0 / (uint32_t)D.groups_per_block);
  }
  // the tile's queries: words first (one thread per row), then coordinates (the workgroup together)
  uint32_t my_len = 0;
  if ((int)threadIdx.x < rows) {
    TileQuery t{};
    if (threadIdx.x < pairs) {
      const uint32_t pk = S.grouped[first + threadIdx.x];
      t.q = pk >> 10;
      const size_t o = (size_t)t.q * max_nprobe + (pk & 1023u);
      t.len = S.probe_len[o];
      const unsigned long long qb = S.qbase[t.q];
      t.keys = (uint64_t)(uintptr_t)rec_keys_of(S, qb);
      t.poss = (uint64_t)(uintptr_t)rec_poss_of(S, qb);
      t.bound = S.bound[t.q];
      if (METRIC == 0) t.qn = S.qnorm[t.q];
    }
    tq[threadIdx.x] = t;
    my_len = t.len;
  }
  // coordinates: the rows x d / 4 float4s of the tile are dealt out over the workgroup, eight independent
  // loads per thread in flight (a row at a time would be a chain of memory latencies per row); which
  // query a row holds is read from the grouped pairs again rather than waited for in LDS
  {
    const int total = rows * d4;
    constexpr int kInFlight = 8, kThreads = kMmWaves * kWave;
    for (int base = (int)threadIdx.x; base < total; base += kInFlight * kThreads) {
      uint32_t pk[kInFlight];
      int row[kInFlight], col[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {
        const int idx = base + u * kThreads;
        row[u] = idx < total ? idx / d4 : rows;
        col[u] = idx - row[u] * d4;
        pk[u] = row[u] < (int)pairs ? S.grouped[first + row[u]] : 0u;
      }
      float4 v[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u)
        v[u] = row[u] < (int)pairs ? reinterpret_cast<const float4 *>(Q + (size_t)(pk[u] >> 10) * D.d)[col[u]]
                                   : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int u = 0; u < kInFlight; ++u)
        if (row[u] < rows) qs[row[u] * qstride + col[u]] = v[u];
    }
  }
  // how far the longest of the tile's snapshots goes (the first wavefront holds the lengths)
  __shared__ uint32_t s_maxlen;
  if (threadIdx.x < kWave) {
    uint32_t m = my_len;
    for (int o = kWave / 2; o > 0; o >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, o));
    if (threadIdx.x == 0) s_maxlen = m;
  }
  __syncthreads();
  uint32_t g_end = (s_maxlen + kWave - 1) / kWave;  // groups any query of the tile wants
  if (g_end > g_begin + seg) g_end = g_begin + seg;  // ... inside this item's segment
  if (g_end > g_have) g_end = g_have;
  // no barrier from here on: the wavefronts only read the tile
  switch (qg) {
    case 1: scan_groups_mm<METRIC, 1>(D, S, list, g_begin, g_end, first_b, qs, tq, st); break;
    case 2: scan_groups_mm<METRIC, 2>(D, S, list, g_begin, g_end, first_b, qs, tq, st); break;
    case 3: scan_groups_mm<METRIC, 3>(D, S, list, g_begin, g_end, first_b, qs, tq, st); break;
    case 4: scan_groups_mm<METRIC, 4>(D, S, list, g_begin, g_end, first_b, qs, tq, st); break;
    case 6: scan_groups_mm<METRIC, 6>(D, S, list, g_begin, g_end, first_b, qs, tq, st); break;
    default: scan_groups_mm<METRIC, 8>(D, S, list, g_begin, g_end, first_b, qs, tq, st); break;
  }
}

void launch_scan_mm(const Dev &D, const ScanShape &sh, int max_nprobe, const float *Q, const SearchScratch &S,
                    hipStream_t s) {
  // above 64 KiB of dynamic LDS a kernel has to be told (wide vectors only); once per kernel and process
  static const bool once = [] {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_scan_mm<0, false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMmLdsMax);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_scan_mm<1, false>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMmLdsMax);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_scan_mm<0, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMmLdsMax);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_scan_mm<1, true>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMmLdsMax);
    return true;
  }();
  (void)once;
  const dim3 grid((unsigned)sh.grid), block((unsigned)sh.threads);
  if (D.scan_steal) {
    if (D.metric == 0) hipLaunchKernelGGL((k_scan_mm<0, true>), grid, block, sh.lds, s, D, max_nprobe, Q, S, sh.tile_q);
    else hipLaunchKernelGGL((k_scan_mm<1, true>), grid, block, sh.lds, s, D, max_nprobe, Q, S, sh.tile_q);
  } else {
    if (D.metric == 0) hipLaunchKernelGGL((k_scan_mm<0, false>), grid, block, sh.lds, s, D, max_nprobe, Q, S, sh.tile_q);
    else hipLaunchKernelGGL((k_scan_mm<1, false>), grid, block, sh.lds, s, D, max_nprobe, Q, S, sh.tile_q);
  }
}

}  // namespace rtams
