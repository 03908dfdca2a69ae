// In-place rearrangement (Rearrangement algorithm of the paper): the blocks of
// one list are made physically contiguous behind the list's first block, so
// that walking the list needs no header jump.  Block t of the chain belongs at
// physical position first + t; whatever sits there is moved out of the way.
//
// The paper exchanges two blocks through a temporary segment and waits twice
// for the blocks involved to be out of use.  Here the exchange is a relocation in two
// steps, each followed by such a wait (a grace period for the searches in
// flight, arranged by the host with events):
//   step 1  every block that occupies a target position is copied to a block
//           taken from the free stack / bump pointer, and its list's table and
//           header links are switched to the copy;
//   step 2  every misplaced block of the list is copied to its target position
//           and the list's table and links are switched;
//   step 3  the positions the list gave up go to the free stack.
// A search sees, for every block, either the old or the new place, and both
// hold the same bytes while it may look.  The number of blocks in use does not
// change; one spare block per displaced occupant is needed meanwhile, and a round
// moves as many blocks as the spare blocks of the moment allow (at least one as
// long as a single block is free: the paper's one temporary segment), so a long
// chain in a nearly full pool is compacted over several rounds instead of not
// at all.  Exceed() keeps holding for the list until its chain is contiguous;
// only a pool without any spare block stalls it, and that is reported.
#include "rtams_launch.h"

namespace rtams {

constexpr int kRearrThreads = 1024;

// exclusive prefix sum of one value per thread; *total receives the sum
__device__ inline uint32_t wg_exclusive_scan(uint32_t v, uint32_t *lds, uint32_t *total) {
  const int tid = threadIdx.x;
  __syncthreads();
  lds[tid] = v;
  __syncthreads();
  for (int o = 1; o < kRearrThreads; o <<= 1) {
    uint32_t a = tid >= o ? lds[tid - o] : 0u;
    __syncthreads();
    lds[tid] += a;
    __syncthreads();
  }
  if (total) *total = lds[kRearrThreads - 1];
  return lds[tid] - v;
}

__device__ inline void finish_list(const Dev &D, int list) {  // Exceed() no longer holds
  D.online[list] = 0;
  if (D.exceed[list]) {
    D.exceed[list] = 0;
    uint32_t e = atomicSub(&D.ctrl->exceed_lists, 1u);
    D.mirror->exceed_lists = e - 1;
  }
}

// ---- plan: which blocks move where.  One workgroup ("GPU single thread
// execution" in the paper; a workgroup here, the work is a few prefix sums).
__global__ __launch_bounds__(kRearrThreads) void k_rearr_plan(Dev D, RearrangeScratch R, int list_arg) {
  __shared__ uint32_t lds[kRearrThreads];
  __shared__ uint32_t s_list, s_free_in_range, s_vict;
  const int tid = threadIdx.x;
  RearrangeHead *H = R.head;

  // the list: the caller's, or the first one for which Exceed() holds
  // (taken in turn: the first exceeding list behind the one handled last, so that a list that is
  // stalled for lack of a spare block does not keep the others waiting)
  __shared__ uint32_t s_wrap;
  const uint32_t after = H->cursor;  // lists below this one come last
  if (tid == 0) { s_list = list_arg >= 0 ? (uint32_t)list_arg : 0xffffffffu; s_wrap = 0xffffffffu; }
  __syncthreads();
  if (list_arg < 0) {
    for (int l = tid; l < D.nlist; l += kRearrThreads)
      if (D.exceed[l]) atomicMin((uint32_t)l >= after ? &s_list : &s_wrap, (uint32_t)l);
    __syncthreads();
    if (tid == 0 && s_list == 0xffffffffu) s_list = s_wrap;
    __syncthreads();
  }
  const int list = (int)s_list;
  if (tid == 0) {
    H->list = list; H->count = 0; H->nvict = 0; H->done = 0;
    H->state = 0;  // nothing owed, unless the code below says otherwise
    D.mirror->rearr_state = 0;
  }
  if (list < 0 || s_list == 0xffffffffu) return;
  const uint32_t nb = D.nblk[list];
  if (nb <= 1) {
    if (tid == 0) finish_list(D, list);
    return;
  }
  const uint32_t b0 = (uint32_t)*table_entry(D, list, 0);
  // positions 1 .. tmax-1 are handled by this round
  uint32_t tmax = nb;
  if (tmax > D.nblocks - b0) tmax = D.nblocks - b0;  // the pool ends before the chain would
  const uint32_t old_cur = D.ctrl->cur_P;

  // moves, in chain order, at most the capacity of the scratch per round
  uint32_t M = 0;
  for (uint32_t t0 = 1; t0 < tmax && M < R.cap; t0 += kRearrThreads) {
    uint32_t t = t0 + tid;
    bool need = t < tmax && (uint32_t)*table_entry(D, list, t) != b0 + t;
    uint32_t tot;
    uint32_t at = M + wg_exclusive_scan(need ? 1u : 0u, lds, &tot);
    if (need && at < R.cap) R.mv_t[at] = t;
    M = M + tot < R.cap ? M + tot : R.cap;
    __syncthreads();
  }
  if (M == 0) {  // already contiguous as far as the pool allows
    if (tid == 0) finish_list(D, list);
    return;
  }
  __syncthreads();
  const uint32_t M_all = M;  // moves this round would make with spare blocks enough
  const uint32_t lo = b0 + 1;  // first target

  // classify what sits at each target
  uint32_t nvict = 0;
  for (uint32_t j0 = 0; j0 < M; j0 += kRearrThreads) {
    uint32_t j = j0 + tid;
    uint32_t kind = 0;
    if (j < M) {
      uint32_t tgt = b0 + R.mv_t[j];
      if (tgt < old_cur) {
        const BlockHeader *h = block_header(D, tgt);
        if (h->owner >= 0) { kind = 2; R.vic_list[j] = h->owner; R.vic_seq[j] = h->seq; }
        else kind = 1;  // on the free stack
      }
      R.kind[j] = kind;
    }
    uint32_t tot;
    uint32_t at = nvict + wg_exclusive_scan(kind == 2 ? 1u : 0u, lds, &tot);
    if (j < M && kind == 2) R.vic_rank[j] = at;
    nvict += tot;
    __syncthreads();
  }

  // The round covers targets up to and including that of its last move.  Every occupant in use needs a
  // spare block; with fewer spare blocks than occupants the round is cut to as many of its first moves
  // as the spare blocks allow (halved until it fits: a shorter round has fewer occupants, a smaller
  // target range and therefore no fewer spare blocks).
  const int ft = D.ctrl->free_top > 0 ? D.ctrl->free_top : 0;
  uint32_t hi, new_cur, t_last;
  for (;;) {  // uniform over the workgroup
    t_last = R.mv_t[M - 1];
    hi = b0 + t_last;  // last target, inclusive
    // how many free-stack entries lie in the target range (they leave the stack), how many occupants in use
    __syncthreads();
    if (tid == 0) { s_free_in_range = 0; s_vict = 0; }
    __syncthreads();
    for (int i = tid; i < ft; i += kRearrThreads) {
      uint32_t b = (uint32_t)D.free_stack[i];
      if (b >= lo && b <= hi) atomicAdd(&s_free_in_range, 1u);
    }
    for (uint32_t j = tid; j < M; j += kRearrThreads)
      if (R.kind[j] == 2) atomicAdd(&s_vict, 1u);
    __syncthreads();
    nvict = s_vict;
    new_cur = hi + 1 > old_cur ? hi + 1 : old_cur;
    const uint32_t spare = (uint32_t)ft - s_free_in_range + (D.nblocks - new_cur);
    if (nvict <= spare) break;
    if (M == 1) {
      // not a single spare block for the first occupant: nothing can move.  Exceed() keeps holding for
      // the list (its chain is as broken as before); the host is told, and the next round looks at
      // another list first.
      if (tid == 0) {
        H->state = 2;
        H->cursor = (uint32_t)list + 1u < (uint32_t)D.nlist ? (uint32_t)list + 1u : 0u;
        D.mirror->rearr_state = 2;
      }
      return;
    }
    M = (M + 1) / 2;
  }
  // from here on the allocator state changes
  // 1. free-stack entries inside the range are dropped, the rest keeps its order
  uint32_t kept = 0;
  for (int i0 = 0; i0 < ft; i0 += kRearrThreads) {
    int i = i0 + tid;
    uint32_t b = i < ft ? (uint32_t)D.free_stack[i] : 0u;
    bool keep = i < ft && !(b >= lo && b <= hi);
    uint32_t tot;
    uint32_t at = kept + wg_exclusive_scan(keep ? 1u : 0u, lds, &tot);
    __syncthreads();  // every entry of this chunk is read before any is written
    if (keep) D.free_stack[at] = (int32_t)b;
    kept += tot;
    __syncthreads();
  }
  // 2. spare blocks for the occupants: from the stack top first, then the bump pointer
  const uint32_t from_stack = nvict < kept ? nvict : kept;
  for (uint32_t j = tid; j < M; j += kRearrThreads)
    if (R.kind[j] == 2) {
      uint32_t r = R.vic_rank[j];
      R.vic_new[j] = r < from_stack ? (uint32_t)D.free_stack[kept - 1 - r] : new_cur + (r - from_stack);
    }
  __syncthreads();
  if (tid == 0) {
    D.ctrl->free_top = (int)(kept - from_stack);
    D.ctrl->cur_P = new_cur + (nvict - from_stack);
    H->count = M;
    H->nvict = nvict;
    // did this round reach the end of what can be placed?  If not, another is owed.
    H->done = M == M_all && t_last + 1 >= tmax ? 1u : 0u;
    H->state = H->done ? 0u : 1u;
    H->cursor = H->done ? ((uint32_t)list + 1u < (uint32_t)D.nlist ? (uint32_t)list + 1u : 0u) : (uint32_t)list;
    D.mirror->rearr_state = H->state;
  }
}

// ---- block copies: whole blocks (header, ids, vectors), 16 bytes per thread
template <int PHASE>
__global__ __launch_bounds__(256) void k_rearr_copy(Dev D, RearrangeScratch R) {
  const RearrangeHead *H = R.head;
  const uint32_t M = H->count;
  if (M == 0) return;
  const int list = H->list;
  const uint32_t b0 = (uint32_t)*table_entry(D, list, 0);
  const uint32_t per = (uint32_t)(D.block_stride / 16);
  const uint64_t work = (uint64_t)M * per;
  for (uint64_t w = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; w < work;
       w += (uint64_t)gridDim.x * blockDim.x) {
    const uint32_t j = (uint32_t)(w / per), o = (uint32_t)(w - (uint64_t)j * per);
    const uint32_t tgt = b0 + R.mv_t[j];
    uint32_t from, to;
    if (PHASE == 1) {
      if (R.kind[j] != 2) continue;
      from = tgt; to = R.vic_new[j];
    } else {
      from = (uint32_t)*table_entry(D, list, R.mv_t[j]); to = tgt;
    }
    const uint4 *src = reinterpret_cast<const uint4 *>(D.blocks + (size_t)from * D.block_stride);
    uint4 *dst = reinterpret_cast<uint4 *>(D.blocks + (size_t)to * D.block_stride);
    dst[o] = src[o];
  }
}

// ---- table switch: phase 1 points the occupants' lists at the copies, phase 2
// points the list at its target positions (remembering what it gives up)
template <int PHASE>
__global__ __launch_bounds__(256) void k_rearr_tables(Dev D, RearrangeScratch R) {
  const RearrangeHead *H = R.head;
  const uint32_t M = H->count;
  const int list = H->list;
  if (M == 0) return;
  const uint32_t b0 = (uint32_t)*table_entry(D, list, 0);
  for (uint32_t j = blockIdx.x * blockDim.x + threadIdx.x; j < M; j += gridDim.x * blockDim.x) {
    if (PHASE == 1) {
      if (R.kind[j] == 2) *table_entry(D, R.vic_list[j], (uint32_t)R.vic_seq[j]) = (int32_t)R.vic_new[j];
    } else {
      int32_t *e = table_entry(D, list, R.mv_t[j]);
      R.old_src[j] = (uint32_t)*e;
      *e = (int32_t)(b0 + R.mv_t[j]);
    }
  }
}

// ---- header links, rebuilt from the tables once those are final
__device__ inline void relink(const Dev &D, int list, uint32_t seq) {
  const uint32_t nb = D.nblk[list];
  const int32_t me = *table_entry(D, list, seq);
  const int32_t prev = seq > 0 ? *table_entry(D, list, seq - 1) : -1;
  const int32_t next = seq + 1 < nb ? *table_entry(D, list, seq + 1) : -1;
  BlockHeader *h = block_header(D, (uint32_t)me);
  h->owner = list;
  h->seq = (int32_t)seq;
  h->prev = prev;
  h->next = next;
  if (prev >= 0) block_header(D, (uint32_t)prev)->next = me;
  if (next >= 0) block_header(D, (uint32_t)next)->prev = me;
}

template <int PHASE>
__global__ __launch_bounds__(256) void k_rearr_links(Dev D, RearrangeScratch R) {
  const RearrangeHead *H = R.head;
  const uint32_t M = H->count;
  const int list = H->list;
  if (M == 0) return;
  for (uint32_t j = blockIdx.x * blockDim.x + threadIdx.x; j < M; j += gridDim.x * blockDim.x) {
    if (PHASE == 1) {
      if (R.kind[j] == 2) relink(D, R.vic_list[j], (uint32_t)R.vic_seq[j]);
    } else {
      relink(D, list, R.mv_t[j]);
    }
  }
}

// ---- release: the places the list gave up go to the free stack
__global__ __launch_bounds__(256) void k_rearr_release(Dev D, RearrangeScratch R) {
  const RearrangeHead *H = R.head;
  const uint32_t M = H->count;
  if (M == 0) return;
  for (uint32_t j = blockIdx.x * blockDim.x + threadIdx.x; j < M; j += gridDim.x * blockDim.x) {
    const uint32_t old = R.old_src[j];
    block_header(D, old)->owner = -1;
    int at = atomicAdd(&D.ctrl->free_top, 1);
    D.free_stack[at] = (int32_t)old;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0 && H->done) finish_list(D, H->list);
}

void launch_rearr_plan(const Dev &D, const RearrangeScratch &R, int list, hipStream_t s) {
  hipLaunchKernelGGL(k_rearr_plan, dim3(1), dim3(kRearrThreads), 0, s, D, R, list);
}
void launch_rearr_step(const Dev &D, const RearrangeScratch &R, int phase, hipStream_t s) {
  const dim3 g_copy(512), g_small(16), b(256);
  if (phase == 1) {
    hipLaunchKernelGGL(k_rearr_copy<1>, g_copy, b, 0, s, D, R);
    hipLaunchKernelGGL(k_rearr_tables<1>, g_small, b, 0, s, D, R);
    hipLaunchKernelGGL(k_rearr_links<1>, g_small, b, 0, s, D, R);
  } else {
    hipLaunchKernelGGL(k_rearr_copy<2>, g_copy, b, 0, s, D, R);
    hipLaunchKernelGGL(k_rearr_tables<2>, g_small, b, 0, s, D, R);
    hipLaunchKernelGGL(k_rearr_links<2>, g_small, b, 0, s, D, R);
  }
}
void launch_rearr_release(const Dev &D, const RearrangeScratch &R, hipStream_t s) {
  hipLaunchKernelGGL(k_rearr_release, dim3(16), dim3(256), 0, s, D, R);
}

}  // namespace rtams
