// Product-quantised lists: the same blocks, chains and allocator, with M code
// bytes per vector in "mv" instead of d floats.  (The paper names IVF-PQ beside
// IVF-Flat as a kind of list its memory blocks hold and leaves the quantiser to
// the textbook: Jegou et al., product quantization for nearest neighbour
// search.)  This file holds what differs on the insertion side and the
// export; the per-request table of sub-scores lives in group.hip, the scan over
// codes in pq_scan.hip.
//
// Layout: groups of 64 vectors as for floats; the chunk is one 32-bit word of 4
// codes, so a wavefront reading word c of a group loads 256 consecutive bytes,
// lane = vector:  word index = (group * M/4 + c) * 64 + lane.
#include "rtams_launch.h"

namespace rtams {

// ---- fill: one wavefront codes sub-space m of a tile of 8 vectors.  Code m of a vector is the
// entry of codebook m nearest to its sub-vector in squared Euclidean distance, in the fixed
// arithmetic of the coarse quantizer (double, one FMA per dimension, in order), ties to the lowest
// entry.  Lane l holds entries l, l + 64, l + 128, l + 192: it reads each of their coordinates once
// for the 8 vectors, keeps its best (distance, entry) per vector, and a butterfly over the
// wavefront leaves the overall best in every lane; lane v then writes the byte of vector v to its
// place (the wavefront of sub-space 0 also writes the ids).  The codebooks are read from a copy
// with the entries innermost, so that the 64 lanes of a load read consecutive floats.
constexpr int kFillVecs = 8;

__global__ __launch_bounds__(256) void k_pq_fill(Dev D, int64_t n, const float *__restrict__ Y,
                                                 const int64_t *__restrict__ ids, int64_t id_base,
                                                 const int32_t *__restrict__ assign,
                                                 const uint32_t *__restrict__ did) {
  const int M = D.pq_m, ds = D.d / M;
  const int lane = threadIdx.x & (kWave - 1);
  // the same for every lane: said so, so that the vectors' coordinates below come through the scalar unit
  const int64_t w = (int64_t)blockIdx.x * (blockDim.x / kWave) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
  const int64_t tiles = (n + kFillVecs - 1) / kFillVecs;
  if (w >= tiles * M) return;  // uniform over the wavefront
  const int m = (int)(w % M);
  const int64_t i0 = (w / M) * kFillVecs;
  const float *cbt = D.codebooks_t + (size_t)m * ds * 256;  // [dimension][entry]: a wavefront's loads are consecutive
  const float *__restrict__ yrow[kFillVecs];
#pragma unroll
  for (int v = 0; v < kFillVecs; ++v) {
    const int64_t i = i0 + v < n ? i0 + v : n - 1;  // the tail of the last tile repeats the last vector
    yrow[v] = Y + (size_t)i * D.d + (size_t)m * ds;
  }
  double acc[kFillVecs][4];
#pragma unroll
  for (int v = 0; v < kFillVecs; ++v)
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[v][u] = 0.0;
  for (int j = 0; j < ds; ++j) {
    double e[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) e[u] = (double)cbt[(size_t)j * 256 + lane + kWave * u];
#pragma unroll
    for (int v = 0; v < kFillVecs; ++v) {
      const double y = (double)yrow[v][j];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const double t = y - e[u];
        acc[v][u] = __builtin_fma(t, t, acc[v][u]);
      }
    }
  }
  int mine = 0;  // lane v ends up with the code of vector v
#pragma unroll
  for (int v = 0; v < kFillVecs; ++v) {
    double best = acc[v][0];
    int code = lane;
#pragma unroll
    for (int u = 1; u < 4; ++u) {  // ascending entries: strict "<" keeps the lower one on a tie
      const bool take = acc[v][u] < best;
      best = take ? acc[v][u] : best;
      code = take ? lane + kWave * u : code;
    }
    for (int o = kWave / 2; o > 0; o >>= 1) {
      const double ob = __shfl_xor(best, o);
      const int oc = __shfl_xor(code, o);
      const bool take = ob < best || (ob == best && oc < code);
      best = take ? ob : best;
      code = take ? oc : code;
    }
    code = best == best ? code : 0;  // no distance compared (a NaN in the sub-vector): nothing beat the first entry
    if (lane == v) mine = code;
  }
  if (lane >= kFillVecs || i0 + lane >= n) return;
  const int64_t i = i0 + lane;
  const int list = assign[i];
  const uint32_t pos = did[i];
  const uint32_t mid = pos / (uint32_t)D.T_m, moff = pos % (uint32_t)D.T_m;
  if (mid >= D.nblk[list]) return;  // the block could not be opened (pool exhausted)
  const uint32_t b = (uint32_t)*table_entry(D, list, mid);
  uint8_t *bytes = reinterpret_cast<uint8_t *>(block_codes(D, b) + code_word_index(D, moff, m / 4));
  bytes[m % 4] = (uint8_t)mine;
  if (m == 0) block_ids(D, b)[moff] = ids ? ids[i] : id_base + i;
}

// ---- export: thread (position, word): un-interleaves 4 codes of one vector
__global__ __launch_bounds__(256) void k_pq_export(Dev D, int list, int64_t n, int64_t *__restrict__ ids,
                                                   uint8_t *__restrict__ codes) {
  const int words = D.pq_m / 4;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n * words) return;
  const int64_t pos = t / words;
  const int c = (int)(t - pos * words);
  const uint32_t mid = (uint32_t)(pos / D.T_m), moff = (uint32_t)(pos % D.T_m);
  const uint32_t b = (uint32_t)*table_entry(D, list, mid);
  if (codes) reinterpret_cast<uint32_t *>(codes)[pos * words + c] = block_codes(D, b)[code_word_index(D, moff, c)];
  if (ids && c == 0) ids[pos] = block_ids(D, b)[moff];
}

// entries innermost: codebooks_t[m][j][c] = codebooks[m][c][j]
__global__ __launch_bounds__(256) void k_pq_transpose(Dev D) {
  const int ds = D.d / D.pq_m;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)256 * D.d) return;
  const int c = (int)(t & 255);
  const int64_t mj = t >> 8;  // m * ds + j
  const int m = (int)(mj / ds), j = (int)(mj - (int64_t)m * ds);
  D.codebooks_t[t] = D.codebooks[((size_t)m * 256 + c) * ds + j];
}

void launch_pq_transpose(const Dev &D, hipStream_t s) {
  hipLaunchKernelGGL(k_pq_transpose, dim3((unsigned)D.d), dim3(256), 0, s, D);
}

void launch_pq_fill(const Dev &D, int64_t n, const float *Y, const int64_t *ids, int64_t id_base,
                    const InsertScratch &S, hipStream_t s) {
  if (n <= 0) return;
  const int64_t waves = (n + kFillVecs - 1) / kFillVecs * D.pq_m;
  hipLaunchKernelGGL(k_pq_fill, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, D, n, Y, ids, id_base,
                     S.assign, S.did);
}

void launch_pq_export(const Dev &D, int list, int64_t n, int64_t *ids, uint8_t *codes, hipStream_t s) {
  if (n <= 0) return;
  const int64_t threads = n * (D.pq_m / 4);
  hipLaunchKernelGGL(k_pq_export, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, D, list, n, ids, codes);
}

}  // namespace rtams
