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
// centroids are split once, when they are set; the vectors of a batch by a
// small kernel in front of the contraction, which then only copies 16-byte
// operands from memory to LDS to the matrix cores.
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
#ifndef RTAMS_COARSE_VB
#define RTAMS_COARSE_VB 2
#endif
// 32-vector blocks per wavefront: 2 (64 x 64 scores, 3 wavefronts per SIMD) or 4 (64 x 128 scores, a quarter
// less LDS traffic per matrix instruction, 2 wavefronts per SIMD; measured: no faster, 28.0 against 28.8 M
// vectors/s in a bulk load of 20 M x 256 over 16,384 centroids)
constexpr int kVB = RTAMS_COARSE_VB;
constexpr int kTileM = 2 * kVB * 32, kTileN = 128, kTileK = 32;  // vectors, centroids, coordinates per step
constexpr int kVH = kTileM / 64;    // 64-row portions of the vectors a thread stages
// an operand row in LDS: the tile's 4 groups of 8 bf16 (16 bytes each), group g of row r at place
// g ^ ((r >> 1) & 3) of the row's 4: the 8 rows that neighbouring lanes read or write then cover all
// 32 banks once, with no padding
constexpr int kRowBytes = (kTileK / 8) * 16;
__device__ inline int lds_place(int row, int g) { return row * kRowBytes + ((g ^ ((row >> 1) & 3)) * 16); }
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

// bf16 halves of rows of d floats: per row and group of 8 coordinates 16 bytes of hi halves then 16 bytes
// of lo halves; coordinates past d are zero, up to whole steps of 32 (D.dgroups groups)
__device__ inline void split_group(const Dev &D, const float *row, int g, u32x4 *out) {
  float4 u = make_float4(0.f, 0.f, 0.f, 0.f), v = u;
  if (g * 8 < D.d) u = *reinterpret_cast<const float4 *>(row + g * 8);
  if (g * 8 + 4 < D.d) v = *reinterpret_cast<const float4 *>(row + g * 8 + 4);
  u32x4 hi, lo;
  split_eight(u, v, hi, lo);
  out[2 * g] = hi;
  out[2 * g + 1] = lo;
}

__global__ __launch_bounds__(256) void k_centroid_split(Dev D) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)D.nlist * D.dgroups) return;
  const int c = (int)(t / D.dgroups), g = (int)(t % D.dgroups);
  split_group(D, D.centroids + (size_t)c * D.d, g, D.csplit + (size_t)c * D.dgroups * 2);
}

// one wavefront per vector of a batch: its split form and, if asked for, its squared norm
__global__ __launch_bounds__(256) void k_split_rows(Dev D, int64_t n, const float *__restrict__ Y,
                                                    u32x4 *__restrict__ split, float *__restrict__ norms) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t i = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (i >= n) return;  // uniform over the wavefront
  const float *row = Y + i * D.d;
  for (int g = lane; g < D.dgroups; g += kWave) split_group(D, row, g, split + (size_t)i * D.dgroups * 2);
  if (!norms) return;
  float nsq = 0.f;
  for (int j = lane; j < D.d; j += kWave) nsq = fmaf(row[j], row[j], nsq);
  for (int o = kWave / 2; o > 0; o >>= 1) nsq += __shfl_xor(nsq, o);
  if (lane == 0) norms[i] = nsq;
}

// ---- approx[i][c] for i < n, c < nlist
template <int METRIC, bool MATRIX>
__global__ __launch_bounds__(kMfmaThreads, kVB == 2 ? 3 : 2) void k_coarse_mfma(Dev D, int64_t n, const u32x4 *__restrict__ ysplit,
                                                              const float *__restrict__ ynorm,
                                                              float *__restrict__ approx, TileCands tc,
                                                              unsigned long long *cursor_to_clear,
                                                              uint32_t *__restrict__ zero, int zero_n) {
  __shared__ __align__(16) unsigned char s_y[2][kTileM * kRowBytes];  // vectors: hi, lo
  __shared__ __align__(16) unsigned char s_c[2][kTileN * kRowBytes];  // centroids: hi, lo
  __shared__ float s_min[kTileM][2];
  __shared__ float s_cn[kTileN];  // |c|^2 of the tile's centroids (0 past the last one), read after the last barrier of the k loop
  __shared__ float s_norm[kTileM];
  __shared__ uint32_t s_cnt[kTileM];
  __shared__ int32_t s_col[kTileM][kTileCands];
  __shared__ float s_val[kTileM][kTileCands];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int wv = wave & 1, wc = wave >> 1;  // wavefront's place in the 2 (vectors) x 2 (centroids) arrangement
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

  if (tid < kTileN) s_cn[tid] = (METRIC == 0 && col0 + tid < D.nlist) ? D.cnorm[col0 + tid] : 0.f;

  floatx16 acc[2][kVB];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < kVB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  // staging: thread t brings group t % 4 (8 consecutive k, 32 bytes of halves) of rows t / 4 and t / 4 + 64
  // of the vectors and of the centroids into registers, one k-tile ahead: the loads of tile t + 1 are in
  // flight while the matrix cores work on tile t out of LDS.  Rows past the last vector or centroid read
  // the last one (their scores are dropped below); the k past d are zero in both split forms.
  const int ld_row = tid / 4, ld_g = tid % 4;
  const u32x4 *srcy[kVH], *srcc[2];
#pragma unroll
  for (int h = 0; h < kVH; ++h) {
    const int64_t r = row0 + ld_row + 64 * h;
    srcy[h] = ysplit + ((size_t)(r < n ? r : n - 1) * D.dgroups + ld_g) * 2;
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int c = col0 + ld_row + 64 * h;
    srcc[h] = D.csplit + ((size_t)(c < D.nlist ? c : D.nlist - 1) * D.dgroups + ld_g) * 2;
  }
  u32x4 stagey[kVH][2], stagec[2][2];  // [64-row portion][hi, lo]
  auto fetch = [&](int k0) {
#pragma unroll
    for (int h = 0; h < kVH; ++h) {
      stagey[h][0] = srcy[h][k0 / 4];
      stagey[h][1] = srcy[h][k0 / 4 + 1];
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      stagec[h][0] = srcc[h][k0 / 4];
      stagec[h][1] = srcc[h][k0 / 4 + 1];
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < d; k0 += kTileK) {
#pragma unroll
    for (int h = 0; h < kVH; ++h) {
      const int at = lds_place(ld_row + 64 * h, ld_g);
      *reinterpret_cast<u32x4 *>(&s_y[0][at]) = stagey[h][0];
      *reinterpret_cast<u32x4 *>(&s_y[1][at]) = stagey[h][1];
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int at = lds_place(ld_row + 64 * h, ld_g);
      *reinterpret_cast<u32x4 *>(&s_c[0][at]) = stagec[h][0];
      *reinterpret_cast<u32x4 *>(&s_c[1][at]) = stagec[h][1];
    }
    __syncthreads();
    if (k0 + kTileK < d) fetch(k0 + kTileK);  // uniform
    // operands of v_mfma_f32_32x32x16_bf16: lane l supplies 8 consecutive k, the group l / 32 of the
    // 16, of row (or column) l % 32; vectors and centroids use the same split of k over the lanes.
    // The centroids are the rows of the product and the vectors its columns, so that a lane ends up
    // with 32 scores of ONE vector per block column and the smallest of them is found in registers.
#pragma unroll
    for (int kk = 0; kk < kTileK / 16; ++kk) {
      const int off = lds_place(lane & 31, kk * 2 + (lane >> 5));  // (block rows start at multiples of 32: same place)
      bf16x8 ch[2], cl[2], yh[kVB], yl[kVB];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int at = (wc * 64 + a * 32) * kRowBytes + off;
        ch[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&s_c[0][at]));
        cl[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&s_c[1][at]));
      }
#pragma unroll
      for (int b = 0; b < kVB; ++b) {
        const int at = (wv * kVB * 32 + b * 32) * kRowBytes + off;
        yh[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&s_y[0][at]));
        yl[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(&s_y[1][at]));
      }
      // the small products first; every accumulator is touched once in 2 kVB instructions
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < kVB; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cl[a], yh[b], acc[a][b], 0, 0, 0);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < kVB; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[a], yl[b], acc[a][b], 0, 0, 0);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < kVB; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[a], yh[b], acc[a][b], 0, 0, 0);
    }
    __syncthreads();
  }

  // result layout of a 32 x 32 block: register r of lane l holds row (r / 4) * 8 + (l / 32) * 4 + r % 4 (a
  // centroid), column l % 32 (a vector); acc[a][b] is the block of centroid block a and vector block b
  auto centroid_of = [&](int a, int r) { return col0 + wc * 64 + a * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r % 4); };
  // scores in place: |c|^2 - 2 <y, c> or - <y, c>; centroids past the last one score +inf
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int c = centroid_of(a, r);
      const bool real = c < D.nlist;
      const float cn = s_cn[c - col0];
#pragma unroll
      for (int b = 0; b < kVB; ++b)
        acc[a][b][r] = real ? (METRIC == 0 ? cn - 2.f * acc[a][b][r] : -acc[a][b][r]) : __builtin_inff();
    }
  if (MATRIX) {
    const bool quads = D.nlist % 4 == 0;  // a lane's 4 consecutive centroids of one vector go out as one 16-byte store
#pragma unroll
    for (int b = 0; b < kVB; ++b) {
      const int64_t i = row0 + wv * kVB * 32 + b * 32 + (lane & 31);
      if (i >= n) continue;
      float *out = approx + (size_t)i * D.nlist;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; r += 4) {
          const int c = centroid_of(a, r);
          if (quads && c + 3 < D.nlist) {
            *reinterpret_cast<float4 *>(out + c) = make_float4(acc[a][b][r], acc[a][b][r + 1], acc[a][b][r + 2], acc[a][b][r + 3]);
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (c + j < D.nlist) out[c + j] = acc[a][b][r + j];
          }
        }
    }
    return;
  }
  // The tile is reduced here: per vector its smallest score and the centroids within the band of it.
  if (tid < kTileM) s_norm[tid] = ynorm[row0 + tid < n ? row0 + tid : n - 1];
  if (tid < kTileM) s_cnt[tid] = 0u;
#pragma unroll
  for (int b = 0; b < kVB; ++b) {  // smallest score of this lane's vector over the wavefront's 64 centroids
    float v = __builtin_inff();
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r) v = fminf(v, acc[a][b][r]);
    v = fminf(v, __shfl_xor(v, 32));  // the other half of the lanes holds the other centroids of the same vector
    if (lane < 32) s_min[wv * kVB * 32 + b * 32 + lane][wc] = v;
  }
  __syncthreads();
  const float cmax = __uint_as_float(D.ctrl->cnorm_max_bits);
#pragma unroll
  for (int b = 0; b < kVB; ++b) {
    const int row = wv * kVB * 32 + b * 32 + (lane & 31);
    // the smallest of the tile plus 2 E of the vector, a little wider than the refinement's (1.02 against
    // 1.01), so that what the refinement asks for is certainly among what is kept here
    const float limit = fminf(s_min[row][0], s_min[row][1]) + coarse_band(D.d, s_norm[row] + cmax) * 1.02f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (acc[a][b][r] <= limit && centroid_of(a, r) < D.nlist) {
          const uint32_t slot = atomicAdd(&s_cnt[row], 1u);
          if (slot < (uint32_t)kTileCands) {
            s_col[row][slot] = centroid_of(a, r);
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
  // the fixed arithmetic of coarse.hip: one double FMA per dimension, dimensions in order; the
  // 16-byte loads run eight chunks ahead of the chain (a load per turn of the chain, waited for each
  // time, made the chain a sequence of trips to memory)
  const float4 *row4 = reinterpret_cast<const float4 *>(D.centroids + (size_t)c * D.d);
  const float4 *y4 = reinterpret_cast<const float4 *>(y);
  const bool l2 = D.metric == 0;
  double acc = 0.0;
  auto chain = [&](const float4 &a, const float4 &b) {
    if (l2) {
      double t = (double)a.x - (double)b.x; acc = __builtin_fma(t, t, acc);
      t = (double)a.y - (double)b.y; acc = __builtin_fma(t, t, acc);
      t = (double)a.z - (double)b.z; acc = __builtin_fma(t, t, acc);
      t = (double)a.w - (double)b.w; acc = __builtin_fma(t, t, acc);
    } else {
      acc = __builtin_fma((double)a.x, (double)b.x, acc);
      acc = __builtin_fma((double)a.y, (double)b.y, acc);
      acc = __builtin_fma((double)a.z, (double)b.z, acc);
      acc = __builtin_fma((double)a.w, (double)b.w, acc);
    }
  };
  int j = 0;
  for (; j + 8 <= D.d4; j += 8) {
    float4 a[8], b[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { a[u] = y4[j + u]; b[u] = row4[j + u]; }
#pragma unroll
    for (int u = 0; u < 8; ++u) chain(a[u], b[u]);
  }
  for (; j < D.d4; ++j) chain(y4[j], row4[j]);
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

static void launch_split_rows(const Dev &D, int64_t n, const float *Y, u32x4 *split, float *norms, hipStream_t s) {
  hipLaunchKernelGGL(k_split_rows, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, s, D, n, Y, split, norms);
}

void launch_coarse_mfma(const Dev &D, int64_t n, const float *Y, u32x4 *split, float *approx,
                        unsigned long long *cursor_to_clear, uint32_t *zero, int zero_n, hipStream_t s) {
  if (n <= 0) return;
  launch_split_rows(D, n, Y, split, nullptr, s);
  const dim3 grid(tile_grid(D, n));
  const TileCands none{};
  if (D.metric == 0)
    hipLaunchKernelGGL((k_coarse_mfma<0, true>), grid, dim3(kMfmaThreads), 0, s, D, n, split, nullptr, approx, none, cursor_to_clear, zero, zero_n);
  else
    hipLaunchKernelGGL((k_coarse_mfma<1, true>), grid, dim3(kMfmaThreads), 0, s, D, n, split, nullptr, approx, none, cursor_to_clear, zero, zero_n);
}

void launch_coarse_tiles(const Dev &D, int64_t n, const float *Y, u32x4 *split, float *norms, const TileCands &tc,
                         hipStream_t s) {
  if (n <= 0) return;
  launch_split_rows(D, n, Y, split, norms, s);
  const dim3 grid(tile_grid(D, n));
  if (D.metric == 0)
    hipLaunchKernelGGL((k_coarse_mfma<0, false>), grid, dim3(kMfmaThreads), 0, s, D, n, split, norms, nullptr, tc, nullptr, nullptr, 0);
  else
    hipLaunchKernelGGL((k_coarse_mfma<1, false>), grid, dim3(kMfmaThreads), 0, s, D, n, split, norms, nullptr, tc, nullptr, nullptr, 0);
}

void launch_assign_refine(const Dev &D, int64_t n, const float *Y, const TileCands &tc, bool reserve,
                          int32_t *assign, uint32_t *did, hipStream_t s) {
  if (n <= 0) return;
  unsigned grid = (unsigned)((n + 3) / 4);
  hipLaunchKernelGGL(k_assign_refine, dim3(grid), dim3(256), 0, s, D, n, Y, tc, reserve ? 1 : 0, assign, did);
}

}  // namespace rtams
