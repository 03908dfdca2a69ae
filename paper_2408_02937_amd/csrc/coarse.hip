// Coarse quantizer: score of every (vector, centroid) pair in the one fixed
// arithmetic that decides list membership and probe choice (IEEE double, one
// fused multiply-add per dimension, dimensions in ascending order), so that the
// integer decisions are reproducible bit for bit.  Insertion algorithm of the
// paper, step "k <- min(c, y_i)", and the first stage of search.
#include "rtams_launch.h"

namespace rtams {

constexpr int kCoarseThreads = 256;

// vectors per workgroup: their coordinates sit in LDS as doubles, 48 KiB at most (the workgroup has 3 KiB of its own)
int coarse_vt(int d) { return d <= 768 ? 8 : d <= 1536 ? 4 : 2; }
// ... and fewer for a small batch: every slot of a tile costs a full chain of fp64 operations per
// centroid whether a vector sits in it or not, and a batch of a few tiles leaves most of the chip
// idle (one workgroup per tile and centroid split).  The largest tile that still yields a
// workgroup per compute unit, else single vectors.
// Every multiply-add takes one coordinate of a vector out of LDS, the same for the whole wavefront,
// and with eight vectors to a thread the four wavefronts of a CU ask LDS for more than it returns
// (measured: 64 x 8,192 x 768 in 65 us, 15 % of the double-precision rate).  So where that rule picks
// eight or four vectors and there are 512 centroids or more, a thread takes half as many vectors
// against TWO centroids: the same number of chains per thread and of workgroups, half the reads of
// LDS per multiply-add (47 us for that batch).
struct CoarseShape {
  int vt;  // vectors of a workgroup's tile
  int nc;  // centroids a thread takes at a time
};
static CoarseShape coarse_shape(const Dev &D, int64_t n) {
  const int64_t max_s = (D.nlist + kCoarseThreads - 1) / kCoarseThreads;
  for (int vt = coarse_vt(D.d); vt > 1; vt /= 2)
    if ((n + vt - 1) / vt * max_s >= 256) {
      if (vt >= 4 && D.nlist >= 2 * kCoarseThreads) return {vt / 2, 2};
      return {vt, 1};
    }
  return {1, 1};
}

// How many workgroups share the centroids of one vector tile, so that a small
// batch still spreads over the chip.
int coarse_splits(const Dev &D, int64_t n, size_t part_cap) {
  const CoarseShape sh = coarse_shape(D, n);
  int64_t tiles = (n + sh.vt - 1) / sh.vt;
  int max_s = (D.nlist + sh.nc * kCoarseThreads - 1) / (sh.nc * kCoarseThreads);
  int64_t want = (1024 + tiles - 1) / tiles;
  int64_t s = want < 1 ? 1 : want;
  if (s > max_s) s = max_s;
  if (part_cap && (size_t)(s * n) > part_cap) s = (int64_t)(part_cap / (size_t)n);
  if (s < 1) s = 1;
  return (int)s;
}

// is score a better than b, ties to the lower index
__device__ inline bool better_pair(int metric, double a, int ia, double b, int ib) {
  if (a != b) return metric == 0 ? (a < b) : (a > b);
  return ia < ib;
}

// One workgroup: VT vectors (converted to double in LDS) against a range of
// centroids, NC centroids per thread at a time (c and c + 256).  ARGMIN selects
// the epilogue: the best centroid of the range per vector, or all scores.
template <int METRIC, int VT, int NC, bool ARGMIN>
__global__ __launch_bounds__(kCoarseThreads) void k_coarse(
    Dev D, int64_t n, const float *__restrict__ Y, int splits, double *__restrict__ scores,
    double *__restrict__ pscore, int32_t *__restrict__ pidx, unsigned long long *cursor_to_clear,
    uint32_t *__restrict__ zero, int zero_n) {
  extern __shared__ double ylds[];  // [VT][d]
  __shared__ double red_s[kCoarseThreads];
  __shared__ int red_i[kCoarseThreads];
  const int d = D.d, d4 = D.d4;
  const int64_t v0 = (int64_t)blockIdx.x * VT;
  const int split = blockIdx.y;
  // per-request counters of the search plan start from zero (no memset node on the stream)
  if (cursor_to_clear && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *cursor_to_clear = 0ull;
  if (zero) {
    const int nthreads = gridDim.x * gridDim.y * kCoarseThreads;
    for (int i = (blockIdx.y * gridDim.x + blockIdx.x) * kCoarseThreads + threadIdx.x; i < zero_n; i += nthreads)
      zero[i] = 0u;
  }

  for (int t = threadIdx.x; t < VT * d; t += kCoarseThreads) {
    int v = t / d, j = t - v * d;
    int64_t row = v0 + v;
    ylds[t] = row < n ? (double)Y[row * d + j] : 0.0;
  }
  __syncthreads();

  // centroid range of this split, in units of one row per thread
  constexpr int kStep = NC * kCoarseThreads;  // centroids the workgroup takes at a time
  const int per = ((D.nlist + splits - 1) / splits + kStep - 1) / kStep * kStep;
  const int c_begin = split * per;
  const int c_end = min(D.nlist, c_begin + per);

  // running best per vector; the sentinel loses against every real score
  const double worst = METRIC == 0 ? __builtin_inf() : -__builtin_inf();
  double best_s[VT];
  int best_i[VT];
#pragma unroll
  for (int v = 0; v < VT; ++v) { best_s[v] = worst; best_i[v] = 0x7fffffff; }

  // The centroids stream in from their transposed copy: chunk j of 64 consecutive centroids is 1 KiB,
  // one 16-byte load per lane.  A thread's chain of multiply-adds is sequential in the coordinates, so
  // what hides the trips to memory is how far ahead of the chain the loads run: four sets of kSet
  // chunks go round, three of them in flight while the fourth is used up (a single query against
  // thousands of centroids is nothing but such chains, a few per CU).
  constexpr int kSet = VT <= 2 && NC == 1 ? 8 : 4;
  const float4 *CT = reinterpret_cast<const float4 *>(D.centroids_t);
  const size_t cstride = (size_t)D.nlist;
  for (int c = c_begin + threadIdx.x; c < c_end; c += kStep) {
    double acc[NC][VT];
#pragma unroll
    for (int e = 0; e < NC; ++e)
#pragma unroll
      for (int v = 0; v < VT; ++v) acc[e][v] = 0.0;
    // (a second centroid past the range reads the last centroid: its scores are dropped below)
    const float4 *col[NC];
#pragma unroll
    for (int e = 0; e < NC; ++e) col[e] = CT + min(c + e * kCoarseThreads, D.nlist - 1);
    auto load_set = [&](float4 (*set)[kSet], int j0) {
#pragma unroll
      for (int e = 0; e < NC; ++e)
#pragma unroll
        for (int u = 0; u < kSet; ++u) set[e][u] = col[e][(size_t)(j0 + u) * cstride];
      __builtin_amdgcn_sched_barrier(0);  // the loads go out here, not where they are used
    };
    // the vectors' coordinates of chunk j, out of LDS
    auto read_y = [&](double (*y)[4], int j) {
#pragma unroll
      for (int v = 0; v < VT; ++v) {
        const double *p = ylds + v * d + 4 * j;
        y[v][0] = p[0]; y[v][1] = p[1]; y[v][2] = p[2]; y[v][3] = p[3];
      }
    };
    auto fma_chunk = [&](int e, const float4 &cv, const double (*y)[4]) {
      const double c0 = (double)cv.x, c1 = (double)cv.y, c2 = (double)cv.z, c3 = (double)cv.w;
#pragma unroll
      for (int v = 0; v < VT; ++v) {
        if (METRIC == 0) {
          double t0 = y[v][0] - c0; acc[e][v] = __builtin_fma(t0, t0, acc[e][v]);
          double t1 = y[v][1] - c1; acc[e][v] = __builtin_fma(t1, t1, acc[e][v]);
          double t2 = y[v][2] - c2; acc[e][v] = __builtin_fma(t2, t2, acc[e][v]);
          double t3 = y[v][3] - c3; acc[e][v] = __builtin_fma(t3, t3, acc[e][v]);
        } else {
          acc[e][v] = __builtin_fma(y[v][0], c0, acc[e][v]);
          acc[e][v] = __builtin_fma(y[v][1], c1, acc[e][v]);
          acc[e][v] = __builtin_fma(y[v][2], c2, acc[e][v]);
          acc[e][v] = __builtin_fma(y[v][3], c3, acc[e][v]);
        }
      }
    };
    // With one or two vectors to a thread a chunk is four or eight dependent multiply-adds, and a trip
    // to LDS in front of each chunk would take longer than they do: the coordinates of the next
    // chunk are asked for before this one is worked on.
    constexpr bool kAhead = VT <= 2;
    auto use_set = [&](const float4 (*set)[kSet], int j0) {
      if (kAhead) {
        double ya[VT][4], yb[VT][4];
        read_y(ya, j0);
#pragma unroll
        for (int u = 0; u < kSet; u += 2) {
          read_y(yb, j0 + u + 1);
#pragma unroll
          for (int e = 0; e < NC; ++e) fma_chunk(e, set[e][u], ya);
          if (u + 2 < kSet) read_y(ya, j0 + u + 2);
#pragma unroll
          for (int e = 0; e < NC; ++e) fma_chunk(e, set[e][u + 1], yb);
        }
      } else {
#pragma unroll
        for (int u = 0; u < kSet; ++u) {
          double y[VT][4];
          read_y(y, j0 + u);  // once for the thread's centroids
#pragma unroll
          for (int e = 0; e < NC; ++e) fma_chunk(e, set[e][u], y);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    constexpr int kRing = 4 * kSet;
    const int d4_main = d4 / kRing * kRing;  // chunks that go through the four sets; the rest one at a time
    if (d4_main) {  // uniform
      float4 s0[NC][kSet], s1[NC][kSet], s2[NC][kSet], s3[NC][kSet];
      load_set(s0, 0);
      load_set(s1, kSet);
      load_set(s2, 2 * kSet);
      int j = 0;
#pragma unroll 1
      for (; j + kRing < d4_main; j += kRing) {
        load_set(s3, j + 3 * kSet);
        use_set(s0, j);
        load_set(s0, j + kRing);
        use_set(s1, j + kSet);
        load_set(s1, j + kRing + kSet);
        use_set(s2, j + 2 * kSet);
        load_set(s2, j + kRing + 2 * kSet);
        use_set(s3, j + 3 * kSet);
      }
      load_set(s3, j + 3 * kSet);
      use_set(s0, j);
      use_set(s1, j + kSet);
      use_set(s2, j + 2 * kSet);
      use_set(s3, j + 3 * kSet);
    }
    for (int j = d4_main; j < d4; ++j) {
      double y[VT][4];
      read_y(y, j);
#pragma unroll
      for (int e = 0; e < NC; ++e) fma_chunk(e, col[e][(size_t)j * cstride], y);
    }
#pragma unroll
    for (int e = 0; e < NC; ++e) {
      const int ce = c + e * kCoarseThreads;
      if (ce >= c_end) break;
      if (ARGMIN) {
#pragma unroll
        for (int v = 0; v < VT; ++v) {
          const bool take = better_pair(METRIC, acc[e][v], ce, best_s[v], best_i[v]);
          best_s[v] = take ? acc[e][v] : best_s[v];
          best_i[v] = take ? ce : best_i[v];
        }
      } else {
#pragma unroll
        for (int v = 0; v < VT; ++v)
          if (v0 + v < n) scores[(size_t)(v0 + v) * D.nlist + ce] = acc[e][v];
      }
    }
  }

  if (ARGMIN) {
#pragma unroll
    for (int v = 0; v < VT; ++v) {
      __syncthreads();
      red_s[threadIdx.x] = best_s[v];
      red_i[threadIdx.x] = best_i[v];
      __syncthreads();
      for (int w = kCoarseThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
          const int ib = red_i[threadIdx.x + w], ia = red_i[threadIdx.x];
          const double sb = red_s[threadIdx.x + w], sa = red_s[threadIdx.x];
          const bool take = better_pair(METRIC, sb, ib, sa, ia);
          red_s[threadIdx.x] = take ? sb : sa;
          red_i[threadIdx.x] = take ? ib : ia;
        }
        __syncthreads();
      }
      if (threadIdx.x == 0 && v0 + v < n) {
        pscore[(size_t)(v0 + v) * splits + split] = red_s[0];
        pidx[(size_t)(v0 + v) * splits + split] = red_i[0] == 0x7fffffff ? -1 : red_i[0];
      }
    }
  }
}

// once per set_centroids: the transposed copy the kernel above streams
__global__ __launch_bounds__(256) void k_centroid_transpose(Dev D) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)D.nlist * D.d4) return;
  const int j = (int)(t / D.nlist), c = (int)(t % D.nlist);  // consecutive threads write consecutive 16 bytes
  reinterpret_cast<float4 *>(D.centroids_t)[t] = reinterpret_cast<const float4 *>(D.centroids)[(size_t)c * D.d4 + j];
}

void launch_centroid_transpose(const Dev &D, hipStream_t s) {
  const int64_t items = (int64_t)D.nlist * D.d4;
  hipLaunchKernelGGL(k_centroid_transpose, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, s, D);
}

template <bool ARGMIN>
static void launch_coarse(const Dev &D, int64_t n, const float *Y, int splits, double *scores,
                          double *pscore, int32_t *pidx, unsigned long long *cursor, uint32_t *zero,
                          int zero_n, hipStream_t s) {
  if (n <= 0) return;
  const CoarseShape sh = coarse_shape(D, n);
  const int vt = sh.vt;
  dim3 grid((unsigned)((n + vt - 1) / vt), (unsigned)splits);
  size_t lds = (size_t)vt * D.d * sizeof(double);
#define RTAMS_GO(M, V, N_) \
  hipLaunchKernelGGL((k_coarse<M, V, N_, ARGMIN>), grid, dim3(kCoarseThreads), lds, s, D, n, Y, splits, \
                     scores, pscore, pidx, cursor, zero, zero_n)
  if (D.metric == 0) {
    if (vt == 8) RTAMS_GO(0, 8, 1); else if (vt == 4 && sh.nc == 2) RTAMS_GO(0, 4, 2); else if (vt == 4) RTAMS_GO(0, 4, 1);
    else if (vt == 2 && sh.nc == 2) RTAMS_GO(0, 2, 2); else if (vt == 2) RTAMS_GO(0, 2, 1); else RTAMS_GO(0, 1, 1);
  } else {
    if (vt == 8) RTAMS_GO(1, 8, 1); else if (vt == 4 && sh.nc == 2) RTAMS_GO(1, 4, 2); else if (vt == 4) RTAMS_GO(1, 4, 1);
    else if (vt == 2 && sh.nc == 2) RTAMS_GO(1, 2, 2); else if (vt == 2) RTAMS_GO(1, 2, 1); else RTAMS_GO(1, 1, 1);
  }
#undef RTAMS_GO
}

void launch_coarse_scores(const Dev &D, int64_t n, const float *Y, double *scores,
                          unsigned long long *cursor_to_clear, uint32_t *zero, int zero_n, hipStream_t s) {
  int splits = coarse_splits(D, n, 0);
  launch_coarse<false>(D, n, Y, splits, scores, nullptr, nullptr, cursor_to_clear, zero, zero_n, s);
}

void launch_coarse_argmin(const Dev &D, int64_t n, const float *Y, int splits, double *pscore,
                          int32_t *pidx, hipStream_t s) {
  launch_coarse<true>(D, n, Y, splits, nullptr, pscore, pidx, nullptr, nullptr, 0, s);
}

}  // namespace rtams
