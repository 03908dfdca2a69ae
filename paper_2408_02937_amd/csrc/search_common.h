// What the kernels of the search path share: monotone key maps, where a query's survivor records
// lie, workgroup-wide selection and sorting in LDS, the fp32 score of a vector against a query,
// and the launch shape of the list scan (the planning kernel needs it as well).
#pragma once
#include <type_traits>
#include "rtams_launch.h"

namespace rtams {

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
// back and shares the sibling's.  Nobody waits for anybody beyond a few bounded second looks.
__device__ inline unsigned long long overflow_take(const SearchScratch &S, unsigned long long want) {
  if (S.ovf_chunks == 0 || want > S.ovf_chunk_cap) return ~0ull;
  // Siblings that race for the request's chunk may hold several free chunks between them for a moment
  // (all but one are handed back at once), and a query of ANOTHER request that looks just then finds
  // every chunk out although one is about to come back: it looks again a bounded number of times
  // before it gives up (a chunk that stays out is held by a request for as long as that request runs).
  uint32_t c = __hip_atomic_load(S.req_chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int round = 0; round < 32 && c == 0; ++round) {
    for (uint32_t e = 0; e < S.ovf_chunks && c == 0; ++e)
      if (atomicCAS(&S.ovf_leased[e], 0u, 1u) == 0u) {
        const uint32_t seen = atomicCAS(S.req_chunk, 0u, e + 1u);
        if (seen == 0u) c = e + 1u;
        else { atomicExch(&S.ovf_leased[e], 0u); c = seen; }
      }
    if (c == 0) c = __hip_atomic_load(S.req_chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // a sibling may have got the last one
    if (c == 0) __builtin_amdgcn_s_sleep(32);
  }
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

// LDS of a selection: two histograms of 256 bins (while one is filled the other is cleared for the
// next pass) and a slot of two 64-bit words per wavefront for the range of the keys.
constexpr int kSelectLdsWords = 2 * 256 + 4 * 16;

// `each(body)` calls body(key) for every key of the calling thread that takes part.  `hist` holds
// kSelectLdsWords words, 8-byte aligned; the workgroup has at most 16 wavefronts.
template <int BITS, typename Each>
__device__ SelectResult wg_radix_select_each(uint32_t k, Each each, uint32_t *hist, uint32_t *bc) {
  typedef typename std::conditional<BITS == 32, unsigned int, unsigned long long>::type Key;  // what the range is reduced in
  // The first digit is the 8 bits that end at the highest bit in which any two keys differ: scores
  // of one query's candidates share sign, exponent and often the first mantissa bits; digits on
  // which every key agrees would make all lanes hit one LDS word (which serialises completely) and
  // decide nothing, and a first digit cut out at a byte boundary often tells only a handful of
  // bins apart.  This way the first pass uses all 256 bins, and a few hundred keys are usually
  // done after one or two.
  uint64_t *range = reinterpret_cast<uint64_t *>(hist + 512);  // per wavefront: {min, max}
  const int lane = (int)(threadIdx.x & (kWave - 1)), wave = (int)(threadIdx.x / kWave);
  __syncthreads();  // whatever used this LDS before is done
  for (int b = threadIdx.x; b < 256; b += blockDim.x) hist[b] = 0;
  {
    Key lo = ~(Key)0, hi = 0;
    each([&](uint64_t key) { lo = (Key)key < lo ? (Key)key : lo; hi = (Key)key > hi ? (Key)key : hi; });
    for (int o = kWave / 2; o > 0; o >>= 1) {
      const Key a = __shfl_xor(lo, o), b = __shfl_xor(hi, o);
      lo = a < lo ? a : lo;
      hi = b > hi ? b : hi;
    }
    if (lane == 0) { range[2 * wave] = (uint64_t)lo; range[2 * wave + 1] = (uint64_t)hi; }
  }
  __syncthreads();
  uint64_t kmin = ~0ull, kmax = 0ull;
  for (int w = 0; w < (int)(blockDim.x / kWave); ++w) {
    const uint64_t a = range[2 * w], b = range[2 * w + 1];
    kmin = a < kmin ? a : kmin;
    kmax = b > kmax ? b : kmax;
  }
  int shift = 0;
  uint64_t prefix = 0, mask = 0;
  {
    const uint64_t diff = kmin ^ kmax;
    const int top = diff ? 63 - __clzll((long long)diff) : -1;  // highest bit in which keys differ
    shift = top < 7 ? 0 : top - 7;
    if (shift > BITS - 8) shift = BITS - 8;
    if (shift + 8 < 64) {
      mask = ~0ull << (shift + 8);
      if (BITS < 64) mask &= (1ull << BITS) - 1ull;
    }
    prefix = kmax & mask;
  }
  uint32_t need = k, c_eq = 0;
  uint32_t *cur = hist, *other = hist + 256;
  for (;;) {
    each([&](uint64_t key) {
      if ((key & mask) == prefix) atomicAdd(&cur[(uint32_t)(key >> shift) & 255u], 1u);
    });
    for (int b = threadIdx.x; b < 256; b += blockDim.x) other[b] = 0;  // for the next pass; last read before the previous barrier
    __syncthreads();
    wg_pick_bin(cur, need, bc);  // ends with a barrier
    const uint32_t dg = bc[0];  // (bc is written again only behind the next barrier)
    need -= bc[1];
    c_eq = bc[2];
    // A digit that overlaps the one before it (the last one, when fewer than 8 bits were left) repeats
    // bits the prefix already holds: only keys that match the prefix were counted, so they agree.
    prefix |= (uint64_t)dg << shift;
    mask |= (uint64_t)255u << shift;
    if (c_eq == need) {  // the whole bin belongs to the k smallest: the lower digits cannot matter
      if (shift > 0) prefix |= (1ull << shift) - 1ull;  // threshold = largest key of the bin
      break;
    }
    if (shift == 0) break;
    shift = shift >= 8 ? shift - 8 : 0;
    uint32_t *t = cur; cur = other; other = t;
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
    // the second key is only looked at where the first ties; four first keys per round of LDS reads
    auto count = [&](int j, uint64_t b1) {
      if (b1 < a1) {
        ++before;
      } else if (b1 == a1) {
        const uint64_t b2 = k2[j];
        before += (b2 < a2 || (b2 == a2 && j < e)) ? 1u : 0u;
      }
    };
    int j = lo;
    for (; j + 4 <= hi; j += 4) {
      const uint64_t b0 = k1[j], b1 = k1[j + 1], b2 = k1[j + 2], b3 = k1[j + 3];
      count(j, b0); count(j + 1, b1); count(j + 2, b2); count(j + 3, b3);
    }
    for (; j < hi; ++j) count(j, k1[j]);
  }
  for (int o = 1; o < S; o <<= 1) before += __shfl_xor(before, o);  // the S lanes of an entry are neighbours in one wavefront
  __syncthreads();  // everybody has read
  if (on && s == 0) { k1[before] = a1; k2[before] = a2; pay[before] = ap; }
  __syncthreads();
}


// ------------------------------------------------------------------ fp32 score
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

// ------------------------------------------- dot products on the matrix cores
// v_mfma_f32_4x4x1 (16 blocks): a wavefront multiplies, block by block, a column of 4 values of A by a
// row of 4 values of B.  Lane l supplies one value of each; component r of the result in lane l is
//   a[lane 4 (l / 4) + r] * b[lane l]
// added to what the component held.  With a = one coordinate of the 64 vectors of a group (lane =
// vector, exactly what the interleaved layout hands to a wavefront) and b = the same coordinate of
// query l % 4, d such instructions leave, in lane l, the inner products of vectors 4 (l / 4) .. + 3 with
// query l % 4: 64 vectors x 4 queries per instruction and coordinate, no data movement in between.
typedef float MfmaAcc __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void mfma_step(MfmaAcc &acc, float x, float y) {
  acc = __builtin_amdgcn_mfma_f32_4x4x1f32(x, y, acc, 0, 0, 0);
}
// a chunk of 4 coordinates into one accumulator, in the order of the coordinates
__device__ __forceinline__ void mfma_chunk(MfmaAcc &acc, const float4 &x, const float4 &y) {
  mfma_step(acc, x.x, y.x);
  mfma_step(acc, x.y, y.y);
  mfma_step(acc, x.z, y.z);
  mfma_step(acc, x.w, y.w);
}
// value of lane 4 (l / 4) + r for every lane l (a move inside each group of four lanes)
template <int R>
__device__ __forceinline__ float quad_broadcast(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), R * 0x55, 0xf, 0xf, true));
}

// ---- norm form of the squared distance.  On the matrix cores a squared distance is scored as
// |x|^2 + |q|^2 - 2 <x, q> (the inner products are the contraction; |x|^2 is accumulated once per
// vector beside it).  That value differs from the direct form sum (x - q)^2 (which is what the bound's
// sample computes and what is returned) by rounding errors that grow with the norms, not with the
// distance:
//   |norm form - direct form| <= slack * (2 v + 3 |q|^2),  slack = 1.01 (4 d + 8) 2^-24,
// for v either of the two values (d roundings for |x|^2, up to 2 d for <x, q> whatever the order of
// its terms, three more for the combination, d + 2 roundings of the direct form; |x|^2 + |q|^2 <=
// 2 |x - q|^2 + 3 |q|^2).  So whoever compares a norm-form score with a limit taken from direct-form
// scores, or the other way round, first raises the limit by that much ("loosened"), and the selection
// scores its finalists again in the direct form: the result is the one the direct form gives.
__device__ inline float norm_form_slack(int d) { return 1.01f * (float)(4 * d + 8) * 5.9604645e-8f; }
__device__ inline float loosened(float v, float slack, float qn) {
  const float r = v + slack * (2.f * fmaxf(v, 0.f) + 3.f * qn) + 1e-30f;
  return r + fabsf(r) * 2.4e-7f;  // the rounding of this very computation
}
__device__ inline float l2_score_of_key(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}
__device__ inline uint32_t loosened_key(uint32_t key, float slack, float qn) {
  if (key == 0xFFFFFFFFu) return key;  // "keep everything"
  return key_of_float(loosened(l2_score_of_key(key), slack, qn) + 0.0f);
}
// which lists a request scores through the norm form: flat float lists under the L2 metric
__device__ __host__ inline bool uses_norm_form(const Dev &D) {
  return D.scan_mfma != 0 && D.metric == 0 && D.pq_m == 0 && D.storage == 0;
}


// ---------------------------------------------------- launch shape of the scan
// Hardware hands consecutive workgroup ids to the 8 XCDs in turn; a workgroup of the scan is up to
// four wavefronts, one work item each.
constexpr uint32_t kXcds = 8;
constexpr int kScanWaves = 4;

// Launch shape of a list scan.  Two kernels share the plan of work items (list, segment, tile of the
// queries probing the list):
//  - vector unit (narrow storage, small requests, or the matrix cores switched off): a workgroup is up
//    to four wavefronts that take four consecutive items, one each, every one with its own tile of up
//    to 8 queries in LDS;
//  - matrix cores (flat float lists, requests of 64 queries or more): a workgroup takes ONE item, its
//    tile of up to 32 queries sits in LDS once, and its four wavefronts share out the item's groups of
//    vectors.  Large tiles are what keeps a hot list from being read once per 8 of the dozens of
//    queries that probe it; the price is registers (3 wavefronts per SIMD instead of 4) and a tile to
//    set up per item, which small requests, whose tiles hold a query or two, do not get back
//    (measured at 1 and 32 queries: 15 to 20 % slower than the vector unit with its partial-distance
//    pruning).
struct ScanShape {
  bool mm;           // the matrix-core kernel
  int tile_q;        // queries of a tile at most
  int min_choice;    // shortest segment the plan may choose: 2 << min_choice groups of 64 vectors
  int items_per_wg;  // items a workgroup takes
  int threads;       // of a workgroup
  int grid;          // workgroups
  size_t lds;        // dynamic LDS bytes of a workgroup
};
constexpr int kMmWaves = 4;            // wavefronts of a workgroup of the matrix-core scan
constexpr int kMmTileMax = 32;         // queries of its tile at most
constexpr int kMmQueryWords = 12;      // 32-bit words of LDS per query of a tile beside its coordinates
constexpr int kMmStageCap = 256;       // survivors a wavefront stages in LDS before it reserves their places
constexpr size_t kMmStageBytes = (size_t)kMmStageCap * 9 + 8 * kMmTileMax;  // keys, positions, rows, and two words per query of the tile
constexpr size_t kMmLdsMax = 160 * 1024 - 1024;  // what a workgroup may take of the CU's 160 KiB
constexpr int kMmMinBatch = 64;        // queries of a request from which the matrix-core scan pays

inline ScanShape scan_shape(const Dev &D, int item_budget) {
  ScanShape sh{};
  sh.mm = D.scan_mfma != 0 && D.storage == 0 && D.pq_m == 0;
  // room for an uneven split of the items over the XCDs
  const int items = item_budget + item_budget / 2;
  if (!sh.mm) {
    const size_t per_wave = (size_t)kScanTileQueries * D.d * sizeof(float);
    int waves = kScanWaves;  // as many (4, 2, 1) as fit their query tiles into 64 KiB of LDS
    while (waves > 1 && per_wave * waves > 65536) waves /= 2;
    sh.tile_q = kScanTileQueries;
    sh.min_choice = 0;
    sh.items_per_wg = waves;
    sh.threads = waves * kWave;
    sh.lds = per_wave * waves;
    sh.grid = ((items + waves - 1) / waves + (int)kXcds - 1) / (int)kXcds * (int)kXcds;
    return sh;
  }
  const size_t row = (size_t)(D.d + 4) * sizeof(float) + kMmQueryWords * 4;  // a query of the tile: coordinates, one float4 of padding, its words
  const size_t stage = kMmWaves * kMmStageBytes;
  int rows = kMmTileMax;
  // two workgroups should fit a CU side by side; a tile is never below 8 queries unless LDS cannot hold that
  while (rows > 8 && row * rows + stage > 64 * 1024) rows /= 2;
  while (rows > 4 && row * rows + stage > kMmLdsMax) rows /= 2;
  sh.tile_q = rows;
  sh.min_choice = 2;  // at least 8 groups to an item, two for every wavefront (measured: 4 and 16 are slower)
  if (D.scan_min_choice >= 0) sh.min_choice = D.scan_min_choice;
  sh.items_per_wg = 1;
  sh.threads = kMmWaves * kWave;
  sh.lds = row * rows + stage;
  sh.grid = (items + (int)kXcds - 1) / (int)kXcds * (int)kXcds;
  return sh;
}

// Workgroup of the planning kernel (k_group).  Two of them fit a CU side by side, so that a request
// of as many queries as the chip has CUs, with its two extra workgroups, still starts all at once
// (with 1024 threads the last two waited for the first to finish: 17 us at 256 queries).
constexpr int kGroupThreads = 512;

}  // namespace rtams
