// Coarse quantizer as a dense contraction on the matrix cores, used when a
// batch is large enough for that to pay (bulk loads, big insertion batches,
// query batches against many centroids): approximate scores of every (vector,
// centroid) pair.
//
// The contraction runs on the bf16 matrix instruction, which is sixteen times
// as fast as the fp32 one, on operands split in two: x = hi + lo + r with
// hi = bf16(x), lo = bf16(x - hi), |r| <= 2^-16 |x|.  Three products,
// hi hi + hi lo + lo hi (each exact in fp32, accumulated in fp32), leave out
// lo lo and the two r terms: at most 3.02 * 2^-16 |x c| per coordinate.  The
// centroids are split once, when they are set; the vectors on their way into
// LDS.
//
// The approximate scores only FILTER.  Which list a vector joins and which
// lists a query probes are decided by the fixed double-precision arithmetic of
// coarse.hip on the few centroids the filter cannot tell apart (refinement
// kernels below and in probe.hip), so the decisions stay bit-exact:
//   approx(i, c) = |c|^2 - 2 <y_i, c>   (L2; |y_i|^2 is the same for every c)
//   approx(i, c) = - <y_i, c>           (IP)            smaller is better
// and |approx - exact| <= E_i = (4 (d + 4) 2^-24 + 4 * 2^-16) (|y_i|^2 + max_c |c|^2):
// with sum_j |y_j c_j| <= (|y|^2 + |c|^2) / 2, the split costs 3.02 * 2^-16 of
// that sum twice over (the factor 2 of the L2 form), the 3 d exact products
// added in fp32 in any order (3.05 d) 2^-24 of it twice over, and the rounding
// of |c|^2 and of the final combination 3 * 2^-24 (|y|^2 + |c|^2).  If m is the
// smallest approximate score of row i, the exact winner lies among the centroids
// with approx <= m + 2 E_i (coarse_band() in rtams_launch.h is that 2 E_i).
//
// For a search the whole score matrix is written (probe selection needs the
// nprobe-th smallest of a row).  For an assignment it is not: each workgroup
// reduces its 128 x 128 tile on the spot to, per row, the tile's smallest score
// and the (up to kTileCands) columns within the band of it; the refinement reads
// those few bytes per (row, tile) instead of the matrix, twice.
#include "rtams_launch.h"

namespace rtams {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kMfmaThreads = 256;  // 4 wavefronts: 2 (rows) x 2 (columns), 64 x 64 results each
constexpr int kTileM = 128, kTileN = 128, kTileK = 32;
// an operand row in LDS: the tile's 4 groups of 8 bf16 (16 bytes each) and 16 bytes of padding, so that
// the rows 8 neighbouring lanes read start 20 banks apart and cover all 32
constexpr int kRowBytes = (kTileK / 8) * 16 + 16;
constexpr int kXcds = 8;  // workgroups go to the chip's 8 dies (each with its own L2) in turn

// the two bf16 halves of a pair of floats, packed as the matrix instruction wants them
__device__ inline uint32_t pack_bf16(float a, float b) {
  bf16x2 p;
  p[0] = (__bf16)a;
  p[1] = (__bf16)b;  // round to nearest even
  return __builtin_bit_cast(uint32_t, p);
}
__device__ inline void split_pair(float a, float b, uint32_t &hi, uint32_t &lo) {
  hi = pack_bf16(a, b);
  lo = pack_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));  // the differences are exact
}
__device__ inline void split_eight(const float4 &u, const float4 &v, u32x4 &hi, u32x4 &lo) {
  uint32_t h[4], l[4];
  split_pair(u.x, u.y, h[0], l[0]);
  split_pair(u.z, u.w, h[1], l[1]);
  split_pair(v.x, v.y, h[2], l[2]);
  split_pair(v.z, v.w, h[3], l[3]);
  hi = u32x4{h[0], h[1], h[2], h[3]};
  lo = u32x4{l[0], l[1], l[2], l[3]};
}

// ---- once per set_centroids: squared norms (fp32) with their maximum, and the
// centroids' split form, per centroid and group of 8 coordinates 16 bytes of hi
// halves then 16 bytes of lo halves (coordinates past d are zero)
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

__global__ __launch_bounds__(256) void k_centroid_split(Dev D) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)D.nlist * D.dgroups) return;
  const int c = (int)(t / D.dgroups), g = (int)(t % D.dgroups);
  const float *row = D.centroids + (size_t)c * D.d;
  float4 u = make_float4(0.f, 0.f, 0.f, 0.f), v = u;
  if (g * 8 < D.d) u = *reinterpret_cast<const float4 *>(row + g * 8);
  if (g * 8 + 4 < D.d) v = *reinterpret_cast<const float4 *>(row + g * 8 + 4);
  u32x4 hi, lo;
  split_eight(u, v, hi, lo);
  D.csplit[2 * t] = hi;
  D.csplit[2 * t + 1] = lo;
}

// ---- approx[i][c] for i < n, c < nlist
template <int METRIC, bool MATRIX>
__global__ __launch_bounds__(kMfmaThreads) void k_coarse_mfma(Dev D, int64_t n, const float *__restrict__ Y,
                                                              float *__restrict__ approx, TileCands tc,
                                                              unsigned long long *cursor_to_clear,
                                                              uint32_t *__restrict__ zero, int zero_n) {
  __shared__ __align__(16) unsigned char s_op[4][kTileM * kRowBytes];  // vectors hi, lo; centroids hi, lo
  __shared__ float s_min[kTileM][2];
  __shared__ float s_norm[kTileM];
  __shared__ uint32_t s_cnt[kTileM];
  __shared__ int32_t s_col[kTileM][kTileCands];
  __shared__ float s_val[kTileM][kTileCands];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int wm = wave & 1, wn = wave >> 1;  // wavefront's place in the 2 x 2 arrangement
  const int d = D.d;

  // per-request counters of the search plan start from zero (no memset node on the stream)
  if (cursor_to_clear && blockIdx.x == 0 && tid == 0) *cursor_to_clear = 0ull;
  if (zero) {
    const int nthreads = gridDim.x * kMfmaThreads;
    for (int i = blockIdx.x * kMfmaThreads + tid; i < zero_n; i += nthreads) zero[i] = 0u;
  }

  // Which tile: consecutive workgroups land on consecutive dies, so die x takes the column tiles
  // x, x + 8, ... and walks the row tiles with them: the split centroids of its column tiles stay in
  // its L2 (2 MiB of 4 for 16,384 centroids of 256 dimensions) while the vectors stream through once.
  const int col_tiles = (D.nlist + kTileN - 1) / kTileN, per_die = (col_tiles + kXcds - 1) / kXcds;
  const int die = blockIdx.x % kXcds, turn = blockIdx.x / kXcds;
  const int col_tile = (turn % per_die) * kXcds + die;
  if (col_tile >= col_tiles) return;  // uniform
  const int64_t row0 = (int64_t)(turn / per_die) * kTileM;
  const int col0 = col_tile * kTileN;

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  // staging: thread t brings group t % 4 (8 consecutive k) of rows t / 4 and t / 4 + 64 of the vectors and
  // of the centroids into registers, one k-tile ahead: the loads of tile t + 1 are in flight while the
  // matrix cores work on tile t out of LDS
  const int ld_row = tid / 4, ld_g = tid % 4;
  float nsq[2] = {0.f, 0.f};  // this thread's share of |y_row|^2
  float4 va[2][2];
  u32x4 vb[2][2];
  auto fetch = [&](int k0) {
    const int k = k0 + ld_g * 8;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int64_t r = row0 + ld_row + 64 * h;
      va[h][0] = va[h][1] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < n && k < d) va[h][0] = *reinterpret_cast<const float4 *>(Y + r * d + k);
      if (r < n && k + 4 < d) va[h][1] = *reinterpret_cast<const float4 *>(Y + r * d + k + 4);
      const int c = col0 + ld_row + 64 * h;
      vb[h][0] = vb[h][1] = u32x4{0u, 0u, 0u, 0u};
      if (c < D.nlist && k < d) {
        const u32x4 *p = D.csplit + ((size_t)c * D.dgroups + k / 8) * 2;
        vb[h][0] = p[0];
        vb[h][1] = p[1];
      }
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < d; k0 += kTileK) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const float4 u = va[h][0], v = va[h][1];
      if (!MATRIX)
        nsq[h] = fmaf(u.x, u.x, fmaf(u.y, u.y, fmaf(u.z, u.z, fmaf(u.w, u.w,
                 fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, nsq[h]))))))));
      u32x4 hi, lo;
      split_eight(u, v, hi, lo);
      const int at = (ld_row + 64 * h) * kRowBytes + ld_g * 16;
      *reinterpret_cast<u32x4 *>(&s_op[0][at]) = hi;
      *reinterpret_cast<u32x4 *>(&s_op[1][at]) = lo;
      *reinterpret_cast<u32x4 *>(&s_op[2][at]) = vb[h][0];
      *reinterpret_cast<u32x4 *>(&s_op[3][at]) = vb[h][1];
    }
    __syncthreads();
    if (k0 + kTileK < d) fetch(k0 + kTileK);  // uniform
    // operands of v_mfma_f32_32x32x16_bf16: lane l supplies 8 consecutive k, the group l / 32 of the
    // 16, of row (or column) l % 32; vectors and centroids use the same split of k over the lanes
#pragma unroll
    for (int kk = 0; kk < kTileK / 16; ++kk) {
      const int off = (lane & 31) * kRowBytes + (kk * 2 + (lane >> 5)) * 16;
      bf16x8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int at = (wm * 64 + a * 32) * kRowBytes + off;
        ah[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&s_op[0][at]));
        al[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&s_op[1][at]));
      }
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int at = (wn * 64 + b * 32) * kRowBytes + off;
        bh[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&s_op[2][at]));
        bl[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&s_op[3][at]));
      }
      // the small products first; every accumulator is touched once in four instructions
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[a], bh[b], acc[a][b], 0, 0, 0);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[a], bl[b], acc[a][b], 0, 0, 0);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[a], bh[b], acc[a][b], 0, 0, 0);
    }
    __syncthreads();
  }

  // result layout: register r of lane l holds row (r / 4) * 8 + (l / 32) * 4 + r % 4, column l % 32 of a
  // 32 x 32 block
  auto row_of = [&](int a, int r) { return wm * 64 + a * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r % 4); };
  if (MATRIX) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int c = col0 + wn * 64 + b * 32 + (lane & 31);
      if (c >= D.nlist) continue;
      const float cn = METRIC == 0 ? D.cnorm[c] : 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t i = row0 + row_of(a, r);
          if (i < n) approx[(size_t)i * D.nlist + c] = METRIC == 0 ? cn - 2.f * acc[a][b][r] : -acc[a][b][r];
        }
    }
    return;
  }
  // The tile is reduced here: per row its smallest score and the columns within the band of it.
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int c = col0 + wn * 64 + b * 32 + (lane & 31);
    const bool real = c < D.nlist;
    const float cn = (METRIC == 0 && real) ? D.cnorm[c] : 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        acc[a][b][r] = real ? (METRIC == 0 ? cn - 2.f * acc[a][b][r] : -acc[a][b][r]) : __builtin_inff();
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {  // |y_row|^2: the four threads that staged a row add up their shares
    float t = nsq[h];
    t += __shfl_xor(t, 1);
    t += __shfl_xor(t, 2);
    if ((tid & 3) == 0) s_norm[ld_row + 64 * h] = t;
  }
  if (tid < kTileM) s_cnt[tid] = 0u;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) {  // smallest score of each row over this wavefront's 64 columns
      float v = fminf(acc[a][0][r], acc[a][1][r]);
      for (int o = 16; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));  // stays inside a half of 32 lanes
      if ((lane & 31) == 0) s_min[row_of(a, r)][wn] = v;
    }
  __syncthreads();
  const float cmax = __uint_as_float(D.ctrl->cnorm_max_bits);
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = row_of(a, r);
      const float tmin = fminf(s_min[row][0], s_min[row][1]);
      // 2 E of the row, a little wider than the refinement's (1.02 against 1.01), so that what the
      // refinement asks for is certainly among what is kept here
      const float band = coarse_band(D.d, s_norm[row] + cmax) * 1.02f;
#pragma unroll
      for (int b = 0; b < 2; ++b)
        if (acc[a][b][r] <= tmin + band) {
          const uint32_t slot = atomicAdd(&s_cnt[row], 1u);
          if (slot < (uint32_t)kTileCands) {
            s_col[row][slot] = col0 + wn * 64 + b * 32 + (lane & 31);
            s_val[row][slot] = acc[a][b][r];
          }
        }
    }
  __syncthreads();
  if (tid < kTileM && row0 + tid < n) {
    const size_t at = (size_t)(row0 + tid) * tc.tiles + col_tile;
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
  // 2 E_i; the norm itself carries a relative error of at most d 2^-24, covered by the factor 1.01
  return coarse_band(D.d, ynorm + __uint_as_float(D.ctrl->cnorm_max_bits)) * 1.01f;
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
  const int64_t items = (int64_t)D.nlist * D.dgroups;
  hipLaunchKernelGGL(k_centroid_split, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, D);
}

int coarse_tiles(const Dev &D) { return (D.nlist + kTileN - 1) / kTileN; }

// one workgroup per (row tile, column tile), the column tiles rounded up to a whole turn of the dies
static unsigned tile_grid(const Dev &D, int64_t n) {
  const int64_t per_die = (coarse_tiles(D) + kXcds - 1) / kXcds;
  return (unsigned)(((n + kTileM - 1) / kTileM) * per_die * kXcds);
}

void launch_coarse_mfma(const Dev &D, int64_t n, const float *Y, float *approx,
                        unsigned long long *cursor_to_clear, uint32_t *zero, int zero_n, hipStream_t s) {
  if (n <= 0) return;
  const dim3 grid(tile_grid(D, n));
  const TileCands none{};
  if (D.metric == 0)
    hipLaunchKernelGGL((k_coarse_mfma<0, true>), grid, dim3(kMfmaThreads), 0, s, D, n, Y, approx, none, cursor_to_clear, zero, zero_n);
  else
    hipLaunchKernelGGL((k_coarse_mfma<1, true>), grid, dim3(kMfmaThreads), 0, s, D, n, Y, approx, none, cursor_to_clear, zero, zero_n);
}

void launch_coarse_tiles(const Dev &D, int64_t n, const float *Y, const TileCands &tc, hipStream_t s) {
  if (n <= 0) return;
  const dim3 grid(tile_grid(D, n));
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
