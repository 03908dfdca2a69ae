// Product-quantised lists: the same blocks, chains and allocator, with M code
// bytes per vector in "mv" instead of d floats.  (The paper names IVF-PQ beside
// IVF-Flat as a kind of list its memory blocks hold and leaves the quantiser to
// the textbook: Jegou et al., product quantization for nearest neighbour
// search.)  This file holds what differs on the insertion side and the
// per-request table of sub-scores; the scan over codes lives with the other
// scan in search.hip.
//
// Layout: groups of 64 vectors as for floats; the chunk is one 32-bit word of 4
// codes, so a wavefront reading word c of a group loads 256 consecutive bytes,
// lane = vector:  word index = (group * M/4 + c) * 64 + lane.
#include "rtams_launch.h"

namespace rtams {

// ---- fill: thread (vector i, sub-space m) finds code m of vector i, the entry of codebook m
// nearest to the sub-vector in squared Euclidean distance, in the fixed arithmetic of the coarse
// quantizer (double, one FMA per dimension, in order), ties to the lowest entry, and writes the
// byte to its place; the thread of sub-space 0 also writes the id.
__global__ __launch_bounds__(256) void k_pq_fill(Dev D, int64_t n, const float *__restrict__ Y,
                                                 const int64_t *__restrict__ ids, int64_t id_base,
                                                 const int32_t *__restrict__ assign,
                                                 const uint32_t *__restrict__ did) {
  const int M = D.pq_m, ds = D.d / M;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n * M) return;
  const int64_t i = t / M;
  const int m = (int)(t - i * M);
  const float *y = Y + i * D.d + (size_t)m * ds;
  const float *cb = D.codebooks + (size_t)m * 256 * ds;
  double best = __builtin_inf();
  int code = 0;
  for (int c = 0; c < 256; ++c) {
    const float *e = cb + (size_t)c * ds;
    double acc = 0.0;
    for (int j = 0; j < ds; ++j) {
      const double u = (double)y[j] - (double)e[j];
      acc = __builtin_fma(u, u, acc);
    }
    const bool take = acc < best;  // strict: ties stay with the lower entry
    best = take ? acc : best;
    code = take ? c : code;
  }
  const int list = assign[i];
  const uint32_t pos = did[i];
  const uint32_t mid = pos / (uint32_t)D.T_m, moff = pos % (uint32_t)D.T_m;
  if (mid >= D.nblk[list]) return;  // the block could not be opened (pool exhausted)
  const uint32_t b = (uint32_t)*table_entry(D, list, mid);
  uint8_t *bytes = reinterpret_cast<uint8_t *>(block_codes(D, b) + code_word_index(D, moff, m / 4));
  bytes[m % 4] = (uint8_t)code;
  if (m == 0) block_ids(D, b)[moff] = ids ? ids[i] : id_base + i;
}

// ---- table of sub-scores of a request: lut[q][m][c] = squared distance (L2) or inner product
// (IP) between sub-vector m of query q and entry c of codebook m, fp32, one FMA chain in the
// order of the dimensions.  One workgroup per (query, sub-space), thread = entry.
__global__ __launch_bounds__(256) void k_pq_lut(Dev D, const float *__restrict__ Q, float *__restrict__ lut) {
  const int M = D.pq_m, ds = D.d / M;
  const int q = blockIdx.x, m = blockIdx.y, c = threadIdx.x;
  const float *y = Q + (size_t)q * D.d + (size_t)m * ds;
  const float *e = D.codebooks + ((size_t)m * 256 + c) * ds;
  float acc = 0.f;
  if (D.metric == 0) {
    for (int j = 0; j < ds; ++j) { const float u = e[j] - y[j]; acc = fmaf(u, u, acc); }
  } else {
    for (int j = 0; j < ds; ++j) acc = fmaf(e[j], y[j], acc);
  }
  lut[((size_t)q * M + m) * 256 + c] = acc;
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

void launch_pq_fill(const Dev &D, int64_t n, const float *Y, const int64_t *ids, int64_t id_base,
                    const InsertScratch &S, hipStream_t s) {
  if (n <= 0) return;
  const int64_t threads = n * D.pq_m;
  hipLaunchKernelGGL(k_pq_fill, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, D, n, Y, ids, id_base,
                     S.assign, S.did);
}

void launch_pq_lut(const Dev &D, int64_t nq, const float *Q, float *lut, hipStream_t s) {
  if (nq <= 0) return;
  hipLaunchKernelGGL(k_pq_lut, dim3((unsigned)nq, (unsigned)D.pq_m), dim3(256), 0, s, D, Q, lut);
}

void launch_pq_export(const Dev &D, int list, int64_t n, int64_t *ids, uint8_t *codes, hipStream_t s) {
  if (n <= 0) return;
  const int64_t threads = n * (D.pq_m / 4);
  hipLaunchKernelGGL(k_pq_export, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, D, list, n, ids, codes);
}

}  // namespace rtams
