// Insertion path (Insertion algorithm of the paper): slot reservation with an
// atomic counter per list, lock-free opening and linking of the blocks that do
// not exist yet, in-place fill in the interleaved layout, and publication of
// the batch together with the Exceed() test.
//
// The paper runs all of this in one thread block and separates "reserve",
// "open" and "fill" with two barriers, which only works while a batch cannot
// need two new blocks for one list.  Here the three phases are stream-ordered
// kernels, so any batch size and any block size work across the whole chip; the
// rule that the block of position did lives at chain index did / T_m, offset
// did % T_m, and that exactly one party opens each new block, is the paper's.
#include "rtams_launch.h"

namespace rtams {

__device__ inline void raise_error(const Dev &D, int code) {
  atomicCAS(&D.ctrl->error, 0, code);
  D.mirror->error = code;
}

// ---- reserve: finish the arg-min over the centroid splits, then take the next
// position of that list ("did = atomicAdd(nl_k, 1)").
__global__ __launch_bounds__(256) void k_reserve(Dev D, int64_t n, int splits,
                                                 const double *__restrict__ pscore,
                                                 const int32_t *__restrict__ pidx, int reserve,
                                                 int32_t *__restrict__ assign,
                                                 uint32_t *__restrict__ did) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  double bs = 0.0;
  int bi = -1;
  for (int s = 0; s < splits; ++s) {
    int ci = pidx[i * splits + s];
    if (ci < 0) continue;
    double cs = pscore[i * splits + s];
    bool better = bi < 0 || (cs != bs ? (D.metric == 0 ? cs < bs : cs > bs) : ci < bi);
    if (better) { bs = cs; bi = ci; }
  }
  if (bi < 0) bi = 0;  // no score compared (a vector with a NaN): nothing was better than the first centroid
  assign[i] = bi;
  if (reserve) did[i] = atomicAdd(&D.reserved_len[bi], 1u);
}

// ---- reservation in input order.  The atomic reservation above hands out the positions of a
// batch inside a list in arrival order, which is any order (Algorithm 2 takes `did` from an
// atomicAdd as well).  This variant gives the vectors of a batch that fall into one list
// consecutive positions in the order in which they stand in the batch, which is what inserting
// them one at a time would do: the lists then hold the same SEQUENCE on every run.  One thread per
// list walks the batch's assignments (every lane of a wavefront reads the same word).
__global__ __launch_bounds__(256) void k_reserve_ordered(Dev D, int64_t n, const int32_t *__restrict__ assign,
                                                         uint32_t *__restrict__ did) {
  const int list = blockIdx.x * blockDim.x + threadIdx.x;
  if (list >= D.nlist) return;
  uint32_t at = D.reserved_len[list];
  const uint32_t before = at;
  for (int64_t i = 0; i < n; ++i)
    if (assign[i] == list) did[i] = at++;
  if (at != before) D.reserved_len[list] = at;
}

// ---- open: one wavefront per list.  Positions visible_len .. reserved_len-1
// were reserved by this batch; every block index in [nblk, ceil(reserved/T_m))
// is opened here: table segments first, then blocks from the free stack or the
// bump pointer ("P[atomicAdd(cur_P, 1)]"), headers linked behind the chain.
__global__ __launch_bounds__(256) void k_open(Dev D) {
  const int lane = threadIdx.x & (kWave - 1);
  const int list = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
  if (list >= D.nlist) return;
  const uint32_t T = (uint32_t)D.T_m;
  const uint32_t newlen = D.reserved_len[list];
  const uint32_t nb_old = D.nblk[list];
  const uint32_t nb_new = (newlen + T - 1) / T;
  if (nb_new <= nb_old) return;  // uniform over the wavefront
  if (D.ctrl->error != 0) return;
  const uint32_t count = nb_new - nb_old;

  // table segments: lane s looks after segment s
  int32_t seg_off = -1;
  bool failed = false;
  if (lane < kTableSegs) {
    seg_off = D.seg_dir[(size_t)list * kTableSegs + lane];
    if (seg_off < 0 && lane >= table_seg(nb_old) && lane <= table_seg(nb_new - 1)) {
      uint32_t sz = (uint32_t)kTableBase << lane;
      uint32_t off = atomicAdd(&D.ctrl->slab_cur, sz);
      if ((uint64_t)off + sz > D.slab_cap) failed = true;
      else { seg_off = (int32_t)off; D.seg_dir[(size_t)list * kTableSegs + lane] = seg_off; }
    }
  }

  // blocks: lane 0 takes `count` of them at once
  int f_old = 0;        // free_top before our pop
  uint32_t avail = 0;   // how many came off the free stack
  uint32_t base = 0;    // first block taken from the bump pointer
  if (lane == 0) {
    f_old = atomicSub(&D.ctrl->free_top, (int)count);
    int got = f_old < 0 ? 0 : (f_old < (int)count ? f_old : (int)count);
    if (got < (int)count) atomicAdd(&D.ctrl->free_top, (int)count - got);  // give back what was not there
    avail = (uint32_t)got;
    uint32_t rem = count - avail;
    if (rem) {
      base = atomicAdd(&D.ctrl->cur_P, rem);
      if ((uint64_t)base + rem > D.nblocks) failed = true;
    }
  }
  if (__any(failed)) {  // backstop only: the host refuses batches that might not fit
    if (lane == 0) raise_error(D, -3);
    return;
  }
  f_old = __shfl(f_old, 0);
  avail = __shfl(avail, 0);
  base = __shfl(base, 0);

  auto block_of = [&](uint32_t jl) -> int32_t {  // jl-th new block of this list
    return jl < avail ? D.free_stack[f_old - 1 - (int)jl] : (int32_t)(base + (jl - avail));
  };
  int32_t old_last = -1;
  if (nb_old > 0) {
    int s = table_seg(nb_old - 1);
    int32_t off = __shfl(seg_off, s);
    old_last = D.slab[off + (nb_old - 1 - table_seg_first(s))];
  }

  for (uint32_t j0 = 0; j0 < count; j0 += kWave) {
    uint32_t jl = j0 + lane;
    bool valid = jl < count;
    uint32_t bi = nb_old + (valid ? jl : 0);  // chain index
    int s = table_seg(bi);
    int32_t off = __shfl(seg_off, s);
    if (valid) {
      int32_t b = block_of(jl);
      BlockHeader *h = block_header(D, (uint32_t)b);
      h->prev = jl > 0 ? block_of(jl - 1) : old_last;
      h->next = jl + 1 < count ? block_of(jl + 1) : -1;
      h->owner = list;
      h->seq = (int32_t)bi;
      h->capacity = (int32_t)T;
      h->size = 0;
      D.slab[off + (bi - table_seg_first(s))] = b;
      if (jl == 0 && old_last >= 0) block_header(D, (uint32_t)old_last)->next = b;
    }
  }
  if (lane == 0) D.nblk[list] = nb_new;
}

// ---- fill: thread (vector i, chunk c) writes chunk c (16 bytes: 4 floats, 8 halves or 16 bytes)
// of vector i to its slot; the thread of chunk 0 also writes the id.
__global__ __launch_bounds__(256) void k_fill(Dev D, int64_t n, const float *__restrict__ Y,
                                              const int64_t *__restrict__ ids, int64_t id_base,
                                              const int32_t *__restrict__ assign,
                                              const uint32_t *__restrict__ did) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n * D.vchunks) return;
  int64_t i = t / D.vchunks;
  int c = (int)(t - i * D.vchunks);
  int list = assign[i];
  uint32_t pos = did[i];
  uint32_t mid = pos / (uint32_t)D.T_m, moff = pos % (uint32_t)D.T_m;
  if (mid >= D.nblk[list]) return;  // the block could not be opened (pool exhausted)
  uint32_t b = (uint32_t)*table_entry(D, list, mid);
  const float4 *y = reinterpret_cast<const float4 *>(Y) + i * D.d4;
  float4 v;
  if (D.storage == 1) {
    const float4 a = y[2 * c], e = y[2 * c + 1];
    v = make_float4(__uint_as_float(pack_halves(a.x, a.y)), __uint_as_float(pack_halves(a.z, a.w)),
                    __uint_as_float(pack_halves(e.x, e.y)), __uint_as_float(pack_halves(e.z, e.w)));
  } else if (D.storage == 2) {
    v = make_float4(__uint_as_float(pack_bytes(y[4 * c])), __uint_as_float(pack_bytes(y[4 * c + 1])),
                    __uint_as_float(pack_bytes(y[4 * c + 2])), __uint_as_float(pack_bytes(y[4 * c + 3])));
  } else {
    v = y[c];
  }
  block_vecs(D, b)[vec_chunk_index(D, moff, c)] = v;
  if (c == 0) block_ids(D, b)[moff] = ids ? ids[i] : id_base + i;
}

// ---- publish: one thread per list makes the batch visible and evaluates
// Exceed() (the equation defining it: vectors appended since the last
// rearrangement, strictly greater than T_m').
__global__ __launch_bounds__(256) void k_publish(Dev D, uint32_t call_seq) {
  int list = blockIdx.x * blockDim.x + threadIdx.x;
  // The allocator's counters are final for this batch (k_open has finished, and every rearrangement
  // round enqueued before it has returned its spare blocks): the host learns the blocks in use.
  if (list == 0) {
    const int32_t f = D.ctrl->free_top;
    const uint32_t in_use = D.ctrl->cur_P - (uint32_t)(f > 0 ? f : 0);
    D.mirror->pool_word = ((unsigned long long)call_seq << 32) | in_use;
  }
  if (list >= D.nlist) return;
  uint32_t newlen = D.reserved_len[list];
  uint32_t old = D.visible_len[list];
  if (newlen == old) return;
  if (D.ctrl->error != 0) {  // the batch is dropped as a whole
    D.reserved_len[list] = old;
    return;
  }
  const uint32_t T = (uint32_t)D.T_m;
  for (uint32_t bi = old / T; bi <= (newlen - 1) / T; ++bi) {
    uint32_t b = (uint32_t)*table_entry(D, list, bi);
    uint32_t sz = newlen - bi * T;
    block_header(D, b)->size = (int32_t)(sz < T ? sz : T);
  }
  uint32_t on = D.online[list] + (newlen - old);
  D.online[list] = on;
  if (D.T_mp > 0 && (int64_t)on > D.T_mp && !D.exceed[list]) {
    D.exceed[list] = 1;
    uint32_t e = atomicAdd(&D.ctrl->exceed_lists, 1u);
    D.mirror->exceed_lists = e + 1;
  }
  uint32_t m = atomicMax(&D.ctrl->max_len, newlen);
  if (newlen > m) D.mirror->max_len = newlen;
  atomicAdd(&D.ctrl->ntotal, (unsigned long long)(newlen - old));
  __threadfence();
  __hip_atomic_store(&D.visible_len[list], newlen, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------- launchers

void launch_reserve(const Dev &D, int64_t n, int splits, const InsertScratch &S, bool reserve,
                    int32_t *assign_out, hipStream_t s) {
  if (n <= 0) return;
  unsigned grid = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(k_reserve, dim3(grid), dim3(256), 0, s, D, n, splits, S.pscore, S.pidx,
                     reserve ? 1 : 0, assign_out ? assign_out : S.assign, S.did);
}

void launch_reserve_ordered(const Dev &D, int64_t n, const InsertScratch &S, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(k_reserve_ordered, dim3((unsigned)((D.nlist + 255) / 256)), dim3(256), 0, s, D, n, S.assign,
                     S.did);
}

void launch_open(const Dev &D, hipStream_t s) {
  unsigned grid = (unsigned)((D.nlist + 3) / 4);
  hipLaunchKernelGGL(k_open, dim3(grid), dim3(256), 0, s, D);
}

void launch_fill(const Dev &D, int64_t n, const float *Y, const int64_t *ids, int64_t id_base,
                 const InsertScratch &S, hipStream_t s) {
  if (n <= 0) return;
  int64_t threads = n * D.vchunks;
  unsigned grid = (unsigned)((threads + 255) / 256);
  hipLaunchKernelGGL(k_fill, dim3(grid), dim3(256), 0, s, D, n, Y, ids, id_base, S.assign, S.did);
}

void launch_publish(const Dev &D, uint32_t call_seq, hipStream_t s) {
  unsigned grid = (unsigned)((D.nlist + 255) / 256);
  hipLaunchKernelGGL(k_publish, dim3(grid), dim3(256), 0, s, D, call_seq);
}

}  // namespace rtams
