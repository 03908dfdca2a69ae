// Coarse quantizer as a dense contraction on the matrix cores, used when a
// batch is large enough for that to pay (bulk loads, big insertion batches,
// query batches against many centroids): approximate scores of every (vector,
// centroid) pair in fp32 with v_mfma_f32_32x32x2_f32.
//
// The approximate scores only FILTER.  Which list a vector joins and which
// lists a query probes are decided by the fixed double-precision arithmetic of
// coarse.hip on the few centroids the filter cannot tell apart (refinement
// kernels below and in probe.hip), so the decisions stay bit-exact:
//   approx(i, c) = |c|^2 - 2 <y_i, c>   (L2; |y_i|^2 is the same for every c)
//   approx(i, c) = - <y_i, c>           (IP)            smaller is better
// and |approx - exact| <= E_i = 4 (d + 4) 2^-24 (|y_i|^2 + max_c |c|^2), a bound
// that covers the rounding of the norms, of the dot product in any summation
// order, and of the final combination.  If m is the smallest approximate score
// of row i, the exact winner lies among the centroids with approx <= m + 2 E_i.
//
// For a search the whole score matrix is written (probe selection needs the
// nprobe-th smallest of a row).  For an assignment it is not: each workgroup
// reduces its 64 x 128 tile on the spot to, per row, the tile's smallest score
// and the (up to kTileCands) columns within the band of it; the refinement reads
// those few bytes per (row, tile) instead of the matrix, twice.
#include "rtams_launch.h"

namespace rtams {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kMfmaThreads = 256;  // 4 wavefronts: 2 (rows) x 2 (columns)
constexpr int kTileM = 64, kTileN = 128, kTileK = 16;
constexpr int kLdsStride = kTileK + 1;  // odd stride: the 32 rows of an operand hit 32 banks

// ---- centroid norms (fp32) and their maximum, once per set_centroids
__global__ __launch_bounds__(256) void k_centroid_norms(Dev D) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= D.nlist) return;
  double acc = 0.0;
  const float *row = D.centroids + (size_t)c * D.d;
  for (int j = 0; j < D.d; ++j) acc = __builtin_fma((double)row[j], (double)row[j], acc);
  float n = (float)acc;
  D.cnorm[c] = n;
  atomicMax(&D.ctrl->cnorm_max_bits, __float_as_uint(n));  // non-negative floats order like their bits
}

// ---- approx[i][c] for i < n, c < nlist
template <int METRIC, bool MATRIX>
__global__ __launch_bounds__(kMfmaThreads) void k_coarse_mfma(Dev D, int64_t n, const float *__restrict__ Y,
                                                              float *__restrict__ approx, TileCands tc,
                                                              unsigned long long *cursor_to_clear,
                                                              uint32_t *__restrict__ zero, int zero_n) {
  __shared__ float sA[kTileM * kLdsStride];
  __shared__ float sB[kTileN * kLdsStride];
  __shared__ float s_min[kTileM][2];
  __shared__ float s_norm[kTileM];
  __shared__ uint32_t s_cnt[kTileM];
  __shared__ int32_t s_col[kTileM][kTileCands];
  __shared__ float s_val[kTileM][kTileCands];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int wm = wave & 1, wn = wave >> 1;  // wavefront's place in the 2 x 2 arrangement
  const int64_t row0 = (int64_t)blockIdx.x * kTileM;
  const int col0 = blockIdx.y * kTileN;
  const int d = D.d;

  // per-request counters of the search plan start from zero (no memset node on the stream)
  if (cursor_to_clear && blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) *cursor_to_clear = 0ull;
  if (zero) {
    const int nthreads = gridDim.x * gridDim.y * kMfmaThreads;
    for (int i = (blockIdx.y * gridDim.x + blockIdx.x) * kMfmaThreads + tid; i < zero_n; i += nthreads) zero[i] = 0u;
  }

  floatx16 acc[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;

  // staging: thread t loads a float4 (4 consecutive k) of one row of the vectors and of two rows of the
  // centroids into registers, one k-tile ahead: the loads of tile t + 1 are in flight while the
  // matrix cores work on tile t out of LDS
  const int ld_row = tid / 4, ld_k = (tid % 4) * 4;  // 64 rows x 16 k per pass
  float nsq = 0.f;  // this thread's share of |y_row|^2
  float4 va, vb[2];
  auto fetch = [&](int k0) {
    const int64_t r = row0 + ld_row;
    va = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r < n && k0 + ld_k < d) va = *reinterpret_cast<const float4 *>(Y + r * d + k0 + ld_k);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = col0 + ld_row + 64 * h;
      vb[h] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (c < D.nlist && k0 + ld_k < d)
        vb[h] = *reinterpret_cast<const float4 *>(D.centroids + (size_t)c * d + k0 + ld_k);
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < d; k0 += kTileK) {
    {
      if (!MATRIX) nsq = fmaf(va.x, va.x, fmaf(va.y, va.y, fmaf(va.z, va.z, fmaf(va.w, va.w, nsq))));
      float *dst = sA + ld_row * kLdsStride + ld_k;
      dst[0] = va.x; dst[1] = va.y; dst[2] = va.z; dst[3] = va.w;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float *dst = sB + (ld_row + 64 * h) * kLdsStride + ld_k;
      dst[0] = vb[h].x; dst[1] = vb[h].y; dst[2] = vb[h].z; dst[3] = vb[h].w;
    }
    __syncthreads();
    if (k0 + kTileK < d) fetch(k0 + kTileK);  // uniform
    // operand layout of v_mfma_f32_32x32x2_f32: lane l supplies A[l % 32][l / 32] and B[l / 32][l % 32]
    const float *pa = sA + (wm * 32 + (lane & 31)) * kLdsStride + (lane >> 5);
    const float *pb = sB + (wn * 64 + (lane & 31)) * kLdsStride + (lane >> 5);
#pragma unroll
    for (int kk = 0; kk < kTileK; kk += 2) {
      const float a = pa[kk];
      const float b0 = pb[kk], b1 = pb[32 * kLdsStride + kk];
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc[1], 0, 0, 0);
    }
    __syncthreads();
  }

  // result layout: register r of lane l holds row (r / 4) * 8 + (l / 32) * 4 + r % 4, column l % 32
  if (MATRIX) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int c = col0 + wn * 64 + b * 32 + (lane & 31);
      if (c >= D.nlist) continue;
      const float cn = METRIC == 0 ? D.cnorm[c] : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t i = row0 + wm * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r % 4);
        if (i < n) approx[(size_t)i * D.nlist + c] = METRIC == 0 ? cn - 2.f * acc[b][r] : -acc[b][r];
      }
    }
    return;
  }
  // The tile is reduced here: per row its smallest score and the columns within the band of it.
  float val[2][16];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int c = col0 + wn * 64 + b * 32 + (lane & 31);
    const bool real = c < D.nlist;
    const float cn = (METRIC == 0 && real) ? D.cnorm[c] : 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      val[b][r] = real ? (METRIC == 0 ? cn - 2.f * acc[b][r] : -acc[b][r]) : __builtin_inff();
  }
  {  // |y_row|^2: the four threads that staged a row add up their shares
    float t = nsq;
    t += __shfl_xor(t, 1);
    t += __shfl_xor(t, 2);
    if ((tid & 3) == 0) s_norm[ld_row] = t;
    if (tid < kTileM) s_cnt[tid] = 0u;
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {  // smallest score of each row over this wavefront's 64 columns
    float v = fminf(val[0][r], val[1][r]);
    for (int o = 16; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));  // stays inside a half of 32 lanes
    if ((lane & 31) == 0) s_min[wm * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r % 4)][wn] = v;
  }
  __syncthreads();
  const float cmax = __uint_as_float(D.ctrl->cnorm_max_bits);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = wm * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r % 4);
    const float tmin = fminf(s_min[row][0], s_min[row][1]);
    // 2 E of the row, a little wider than the refinement's (1.02 against 1.01), so that what the
    // refinement asks for is certainly among what is kept here
    const float band = 8.f * (float)(D.d + 4) * 5.9604645e-8f * (s_norm[row] + cmax) * 1.02f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
      if (val[b][r] <= tmin + band) {
        const uint32_t slot = atomicAdd(&s_cnt[row], 1u);
        if (slot < (uint32_t)kTileCands) {
          s_col[row][slot] = col0 + wn * 64 + b * 32 + (lane & 31);
          s_val[row][slot] = val[b][r];
        }
      }
  }
  __syncthreads();
  if (tid < kTileM && row0 + tid < n) {
    const size_t at = (size_t)(row0 + tid) * tc.tiles + blockIdx.y;
    tc.tmin[at] = fminf(s_min[tid][0], s_min[tid][1]);
    tc.cnt[at] = s_cnt[tid];
#pragma unroll
    for (int j = 0; j < kTileCands; ++j) {
      tc.col[at * kTileCands + j] = s_col[tid][j];
      tc.val[at * kTileCands + j] = s_val[tid][j];
    }
  }
}

// ---- refinement of the assignment: one wavefront per vector.  The smallest
// approximate score of the row is the smallest of its tiles' minima; the
// centroids within the error band of it (from the tiles' kept columns; from all
// 128 columns of a tile that had more in the band than it could keep) are
// scored in the fixed double arithmetic and the best is taken, ties to the
// lowest index; then the next position of the list ("did = atomicAdd(nl_k, 1)").
__device__ inline double exact_score(const Dev &D, const float *__restrict__ y, int c) {
  // the fixed arithmetic of coarse.hip: one double FMA per dimension, dimensions in order
  // (loaded four at a time)
  const float4 *row4 = reinterpret_cast<const float4 *>(D.centroids + (size_t)c * D.d);
  const float4 *y4 = reinterpret_cast<const float4 *>(y);
  double acc = 0.0;
  if (D.metric == 0) {
    for (int j = 0; j < D.d4; ++j) {
      const float4 a = y4[j], b = row4[j];
      double t = (double)a.x - (double)b.x; acc = __builtin_fma(t, t, acc);
      t = (double)a.y - (double)b.y; acc = __builtin_fma(t, t, acc);
      t = (double)a.z - (double)b.z; acc = __builtin_fma(t, t, acc);
      t = (double)a.w - (double)b.w; acc = __builtin_fma(t, t, acc);
    }
  } else {
    for (int j = 0; j < D.d4; ++j) {
      const float4 a = y4[j], b = row4[j];
      acc = __builtin_fma((double)a.x, (double)b.x, acc);
      acc = __builtin_fma((double)a.y, (double)b.y, acc);
      acc = __builtin_fma((double)a.z, (double)b.z, acc);
      acc = __builtin_fma((double)a.w, (double)b.w, acc);
    }
  }
  return acc;
}

__device__ inline float error_band(const Dev &D, float ynorm) {
  const float cmax = __uint_as_float(D.ctrl->cnorm_max_bits);
  // 2 E_i with E_i = 4 (d + 4) 2^-24 (|y|^2 + max |c|^2); the norm itself carries a relative
  // error of at most d 2^-24, covered by the factor 1.01
  return 8.f * (float)(D.d + 4) * 5.9604645e-8f * (ynorm + cmax) * 1.01f;
}

__global__ __launch_bounds__(256) void k_assign_refine(Dev D, int64_t n, const float *__restrict__ Y,
                                                       TileCands tc, int reserve,
                                                       int32_t *__restrict__ assign,
                                                       uint32_t *__restrict__ did) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t i = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (i >= n) return;  // uniform over the wavefront
  const float *y = Y + i * D.d;
  const float *tmin = tc.tmin + (size_t)i * tc.tiles;
  float yn = 0.f, m = __builtin_inff();
  for (int j = lane; j < D.d; j += kWave) yn = fmaf(y[j], y[j], yn);
  for (int t = lane; t < tc.tiles; t += kWave) m = fminf(m, tmin[t]);
  for (int o = kWave / 2; o > 0; o >>= 1) {
    yn += __shfl_xor(yn, o);
    m = fminf(m, __shfl_xor(m, o));
  }
  const float limit = m + error_band(D, yn);
  const bool l2 = D.metric == 0;
  double best_s = l2 ? __builtin_inf() : -__builtin_inf();
  int best_c = 0x7fffffff;
  auto offer = [&](int c) {
    const double s = exact_score(D, y, c);
    const bool take = s != best_s ? (l2 ? s < best_s : s > best_s) : c < best_c;
    best_s = take ? s : best_s;
    best_c = take ? c : best_c;
  };
  for (int t0 = 0; t0 < tc.tiles; t0 += kWave) {
    const int t = t0 + lane;
    const size_t at = (size_t)i * tc.tiles + t;
    const bool near = t < tc.tiles && tmin[t] <= limit;
    const uint32_t cnt = near ? tc.cnt[at] : 0u;
    if (near && cnt <= (uint32_t)kTileCands)  // the tile kept all its columns within the band: one lane takes them
      for (uint32_t j = 0; j < cnt; ++j)
        if (tc.val[at * kTileCands + j] <= limit) offer(tc.col[at * kTileCands + j]);
    // a tile with more columns in the band than it could keep: all its columns, shared out over the lanes
    unsigned long long crowded = __ballot(near && cnt > (uint32_t)kTileCands);
    while (crowded) {  // uniform
      const int tt = t0 + __ffsll((long long)crowded) - 1;
      crowded &= crowded - 1;
      for (int c = tt * kTileN + lane; c < (tt + 1) * kTileN && c < D.nlist; c += kWave) offer(c);
    }
  }
  for (int o = kWave / 2; o > 0; o >>= 1) {
    const double s = __shfl_xor(best_s, o);
    const int c = __shfl_xor(best_c, o);
    const bool take = s != best_s ? (l2 ? s < best_s : s > best_s) : c < best_c;
    best_s = take ? s : best_s;
    best_c = take ? c : best_c;
  }
  if (best_c == 0x7fffffff) best_c = 0;  // no score compared (a vector with a NaN): nothing was better than the first centroid
  if (lane == 0) {
    assign[i] = best_c;
    if (reserve) did[i] = atomicAdd(&D.reserved_len[best_c], 1u);
  }
}

void launch_centroid_norms(const Dev &D, hipStream_t s) {
  hipLaunchKernelGGL(k_centroid_norms, dim3((unsigned)((D.nlist + 255) / 256)), dim3(256), 0, s, D);
}

void launch_coarse_mfma(const Dev &D, int64_t n, const float *Y, float *approx,
                        unsigned long long *cursor_to_clear, uint32_t *zero, int zero_n, hipStream_t s) {
  if (n <= 0) return;
  dim3 grid((unsigned)((n + kTileM - 1) / kTileM), (unsigned)((D.nlist + kTileN - 1) / kTileN));
  const TileCands none{};
  if (D.metric == 0)
    hipLaunchKernelGGL((k_coarse_mfma<0, true>), grid, dim3(kMfmaThreads), 0, s, D, n, Y, approx, none, cursor_to_clear, zero, zero_n);
  else
    hipLaunchKernelGGL((k_coarse_mfma<1, true>), grid, dim3(kMfmaThreads), 0, s, D, n, Y, approx, none, cursor_to_clear, zero, zero_n);
}

int coarse_tiles(const Dev &D) { return (D.nlist + kTileN - 1) / kTileN; }

void launch_coarse_tiles(const Dev &D, int64_t n, const float *Y, const TileCands &tc, hipStream_t s) {
  if (n <= 0) return;
  dim3 grid((unsigned)((n + kTileM - 1) / kTileM), (unsigned)tc.tiles);
  if (D.metric == 0)
    hipLaunchKernelGGL((k_coarse_mfma<0, false>), grid, dim3(kMfmaThreads), 0, s, D, n, Y, nullptr, tc, nullptr, nullptr, 0);
  else
    hipLaunchKernelGGL((k_coarse_mfma<1, false>), grid, dim3(kMfmaThreads), 0, s, D, n, Y, nullptr, tc, nullptr, nullptr, 0);
}

void launch_assign_refine(const Dev &D, int64_t n, const float *Y, const TileCands &tc, bool reserve,
                          int32_t *assign, uint32_t *did, hipStream_t s) {
  if (n <= 0) return;
  unsigned grid = (unsigned)((n + 3) / 4);
  hipLaunchKernelGGL(k_assign_refine, dim3(grid), dim3(256), 0, s, D, n, Y, tc, reserve ? 1 : 0, assign, did);
}

}  // namespace rtams
