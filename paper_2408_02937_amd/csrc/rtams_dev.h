// Device-side view of the pool: layout constants, block format, block table.
// Internal to the library; nothing here is part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rtams {

constexpr int kWave = 64;            // gfx950 wavefront
constexpr int kHeaderBytes = 128;    // block header, padded so ids and vectors stay line aligned
constexpr int kTableBase = 32;       // entries of a list's first block-table segment
constexpr int kTableSegs = 20;       // segment s holds kTableBase << s entries
constexpr int kMaxK = 1024;
constexpr int kMaxNprobe = 1024;

// Header of a memory block ("mh" of the paper: previous / next header and block
// info), followed inside the block by the id list "ml" and the vectors "mv".
struct BlockHeader {
  int32_t prev;      // physical block before this one in the chain, -1 at the head
  int32_t next;      // physical block after this one, -1 at the tail
  int32_t owner;     // list that owns the block, -1 when free
  int32_t seq;       // position in the owner's chain
  int32_t capacity;  // T_m
  int32_t size;      // vectors visible in this block
  int32_t pad[26];
};
static_assert(sizeof(BlockHeader) == kHeaderBytes, "header size");

// Control words shared by all kernels (one cache line each for the hot ones).
struct Ctrl {
  uint32_t cur_P;            // bump pointer of the central pool
  uint32_t pad0[31];
  int32_t free_top;          // number of entries on the free stack
  uint32_t pad1[31];
  uint32_t slab_cur;         // bump pointer of the block-table slab
  uint32_t pad2[31];
  int32_t error;             // sticky rtams_status raised by a kernel
  uint32_t exceed_lists;     // lists for which Exceed() holds
  unsigned long long ntotal; // vectors visible
  uint32_t max_len;          // longest visible list
  uint32_t cnorm_max_bits;   // largest squared centroid norm, as float bits
  int32_t search_error;      // rtams_status raised by a kernel of a search (scratch too small): inserts do not look at it
  uint32_t pad3[25];
};

// Words the device writes straight into pinned host memory, so the host can
// read them without synchronising.
struct HostMirror {
  volatile int32_t error;
  volatile uint32_t exceed_lists;
  volatile uint32_t max_len;
  volatile int32_t search_error;
  volatile uint32_t rearr_state;  // of the last rearrangement round: 0 done, 1 another round owed, 2 stalled for lack of a spare block
  // written by every publication, in one store: (number of the last insertion call published << 32) | blocks in
  // use after it.  The host takes from it how many blocks are left without waiting for the data stream.
  volatile unsigned long long pool_word;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct Dev {
  int32_t d, nlist, metric, T_m;
  int32_t pq_m;             // 0: flat lists; M > 0: product-quantiser codes, M bytes per vector
  int32_t scan_mfma;        // flat float lists: the scan's dot products run on the matrix cores (set per request)
  int32_t scan_steal;       // a long scan on the matrix cores: XCDs that are done take items of the others (set per request)
  int32_t scan_min_choice;  // shortest segment the plan may choose, as a power of two of pairs of groups (-1: the kernel's default; set per request)
  int32_t scan_byte_weight; // cost of reading a group of a list, in queries' worth of arithmetic (0: the default; set per request)
  int32_t d4;               // d / 4
  int32_t storage;          // what flat lists keep of a coordinate: 0 float, 1 half, 2 byte
  int32_t vchunks;          // 16-byte chunks of a stored vector: d / 4, d / 8 or d / 16
  int32_t groups_per_block; // T_m / 64
  uint32_t nblocks;         // |P|
  uint32_t slab_cap;        // entries in the table slab
  int64_t T_mp;             // rearrangement threshold
  uint64_t block_stride;    // bytes
  uint32_t ids_off;         // byte offset of the id list inside a block
  uint32_t vec_off;         // byte offset of the vectors inside a block
  char *blocks;
  Ctrl *ctrl;
  HostMirror *mirror;       // pinned host memory, device-visible
  float *centroids;         // [nlist][d]
  float *centroids_t;       // the same numbers as [d / 4][nlist] chunks of 4 coordinates: chunk j of consecutive centroids side by side
  float *cnorm;             // [nlist] squared norms of the centroids (fp32)
  u32x4 *csplit;            // [nlist][dgroups][2] the centroids as bf16 halves: per group of 8 coordinates the 8 hi, then the 8 lo
  int32_t dgroups;          // groups of 8 coordinates of a split row, padded with zeros to whole steps of 32 coordinates: 4 ceil(d / 32)
  float *codebooks;         // [pq_m][256][d / pq_m] (product-quantised lists only)
  float *codebooks_t;       // the same with the entries innermost: [pq_m][d / pq_m][256] (for coding inserted vectors)
  uint32_t *reserved_len;   // [nlist] next free position (atomicAdd target)
  uint32_t *visible_len;    // [nlist] length searches may read
  uint32_t *online;         // [nlist] vectors since the last rearrangement
  uint32_t *nblk;           // [nlist] blocks in the chain
  uint8_t *exceed;          // [nlist] Exceed() holds
  int32_t *seg_dir;         // [nlist][kTableSegs] slab offset of each table segment, -1 unset
  int32_t *slab;            // block-table entries
  int32_t *free_stack;      // [nblocks]
  int32_t *mark;            // [nblocks] scratch for validation
};

// ---- block table: a growable array per list, made of doubling segments ----
__host__ __device__ inline int table_seg(uint32_t i) {
  uint32_t v = i / kTableBase + 1;
#if defined(__HIP_DEVICE_COMPILE__)
  return 31 - __clz((int)v);
#else
  int s = 0;
  while (v >>= 1) ++s;
  return s;
#endif
}
__host__ __device__ inline uint32_t table_seg_first(int s) {
  return (uint32_t)kTableBase * ((1u << s) - 1u);
}

__device__ inline int32_t *table_entry(const Dev &D, int list, uint32_t i) {
  int s = table_seg(i);
  int32_t off = D.seg_dir[(size_t)list * kTableSegs + s];
  return D.slab + off + (i - table_seg_first(s));
}
// The same in its two dependent steps, for callers that want the first on its way early: where the
// table segment of entry i starts (the word exists for every list and segment), then the entry
// (which exists only below the list's number of blocks).
__device__ inline int32_t table_dir(const Dev &D, int list, uint32_t i) {
  return D.seg_dir[(size_t)list * kTableSegs + table_seg(i)];
}
__device__ inline int32_t *table_entry_at(const Dev &D, int32_t dir, uint32_t i) {
  return D.slab + dir + (i - table_seg_first(table_seg(i)));
}

// A vector's place in the pool as one 32-bit number (block * T_m + place in the block; the pool holds
// at most 2^32 places, which rtams_create checks): what a search keeps of a surviving candidate, so
// that whoever needs its id or its coordinates later goes straight to the block.  The block stays
// what it was until the request has finished: a rearrangement waits for the requests in flight
// before it reuses a block.
__device__ inline uint32_t slot_of(const Dev &D, uint32_t b, uint32_t place) { return b * (uint32_t)D.T_m + place; }

__device__ inline BlockHeader *block_header(const Dev &D, uint32_t b) {
  return reinterpret_cast<BlockHeader *>(D.blocks + (size_t)b * D.block_stride);
}
__device__ inline int64_t *block_ids(const Dev &D, uint32_t b) {
  return reinterpret_cast<int64_t *>(D.blocks + (size_t)b * D.block_stride + D.ids_off);
}
__device__ inline float4 *block_vecs(const Dev &D, uint32_t b) {
  return reinterpret_cast<float4 *>(D.blocks + (size_t)b * D.block_stride + D.vec_off);
}

// Product-quantised lists keep the same shape with 4 codes (one 32-bit word) as the chunk:
// word index of codes 4c..4c+3 of the vector at offset moff.
__device__ inline uint32_t *block_codes(const Dev &D, uint32_t b) {
  return reinterpret_cast<uint32_t *>(D.blocks + (size_t)b * D.block_stride + D.vec_off);
}
__device__ inline size_t code_word_index(const Dev &D, uint32_t moff, int c) {
  uint32_t group = moff / kWave, lane = moff % kWave;
  return ((size_t)group * (D.pq_m / 4) + c) * kWave + lane;
}

// Interleaved vector layout inside a block (the paper's equation for "mv",
// re-derived for 64-wide wavefronts): vectors are taken in groups of 64; inside
// a group, chunk c (16 bytes: dimensions 4c..4c+3 of floats, 8c..8c+7 of halves,
// 16c..16c+15 of bytes) of the 64 vectors is contiguous, one float4 per vector.
// A wavefront reading chunk c of a group loads 1 KiB of consecutive memory,
// lane = vector.
__device__ inline size_t vec_chunk_index(const Dev &D, uint32_t moff, int c) {
  uint32_t group = moff / kWave, lane = moff % kWave;
  return ((size_t)group * D.vchunks + c) * kWave + lane;
}

// ---- narrow storage: a 16-byte chunk holds 8 halves or 16 bytes.  piece s of a chunk is the
// float4 of its dimensions 4s..4s+3 (2 pieces of halves, 4 of bytes).
typedef _Float16 Half2 __attribute__((ext_vector_type(2)));
template <int ST>
__device__ __forceinline__ float4 chunk_piece(const float4 &raw, int s) {
  if (ST == 1) {
    const Half2 a = __builtin_bit_cast(Half2, s == 0 ? raw.x : raw.z);
    const Half2 b = __builtin_bit_cast(Half2, s == 0 ? raw.y : raw.w);
    return make_float4((float)a.x, (float)a.y, (float)b.x, (float)b.y);
  } else if (ST == 2) {
    const uint32_t w = __float_as_uint(s == 0 ? raw.x : s == 1 ? raw.y : s == 2 ? raw.z : raw.w);
    return make_float4((float)(w & 255u), (float)((w >> 8) & 255u), (float)((w >> 16) & 255u), (float)(w >> 24));
  }
  return raw;
}
constexpr int pieces_of(int storage) { return storage == 1 ? 2 : storage == 2 ? 4 : 1; }
// the conversions on the way in: IEEE round to nearest even (overflow to infinity) for halves;
// nearest integer, ties to even, clamped to 0..255 for bytes (fmaxf drops a NaN)
__device__ __forceinline__ uint32_t pack_halves(float lo, float hi) {
  Half2 h;
  h.x = (_Float16)lo;
  h.y = (_Float16)hi;
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ uint32_t byte_of(float f) { return (uint32_t)fminf(fmaxf(__builtin_rintf(f), 0.f), 255.f); }
__device__ __forceinline__ uint32_t pack_bytes(const float4 &v) {
  return byte_of(v.x) | (byte_of(v.y) << 8) | (byte_of(v.z) << 16) | (byte_of(v.w) << 24);
}

}  // namespace rtams
