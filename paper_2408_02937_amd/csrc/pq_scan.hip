// The scan of product-quantised lists: per query, the table of sub-scores in LDS, the codes of its
// probed lists looked up in it.
#include "search_common.h"

namespace rtams {

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
      uint32_t len[kPqUnits], slot0[kPqUnits], v[kPqUnits];
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
        slot0[j] = slot_of(D, blk, (g % gpb) * kWave + (uint32_t)lane);
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
            rp[slot] = slot0[j];
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
            my_pos[slot] = slot0[j];
          }
          staged += (uint32_t)__popcll(mask[j]);
        }
      }
    }
  }
  if (staged) pq_flush(S, q, base, my_key, my_pos, staged, lane);
}


void launch_pq_scan(const Dev &D, int64_t nq, int nprobe, int max_nprobe, int item_budget,
                    const SearchScratch &S, hipStream_t s) {
  if (nq <= 0) return;
  // parts per query, from the request's budget of work items: 32 items' worth to a workgroup
  int parts = (int)(item_budget / (nq * 32));
  parts = parts < 1 ? 1 : (parts > 64 ? 64 : parts);
  const size_t lds = (size_t)D.pq_m * 256 * sizeof(float);
  if (lds > 48 * 1024)  // with the kernel's own 8 KiB this passes the default limit of a workgroup
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_pq_scan),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(k_pq_scan, dim3((unsigned)(nq * parts)), dim3(kPqScanThreads), lds, s, D, nprobe,
                     max_nprobe, parts, S);
}

}  // namespace rtams
