// Internal definitions shared by the translation units of libskv (host + device).
#ifndef SKV_INTERNAL_H
#define SKV_INTERNAL_H

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "skv.h"

#define SKV_HD __host__ __device__

// ---- flattened tree as the kernels see it -------------------------------------------------
// Blocks of one node are contiguous in every per-block array ("flat block index").
// Node 0 is the root (no blocks).  A node's children are found through an open-addressed
// table keyed by a 64-bit hash of the child's whole first block; a hit is always confirmed
// by comparing the 16 tokens, so results never depend on the hash.
struct SkvNode {       // 16 bytes
  int32_t first;       // flat index of the node's first block
  int32_t n_blocks;    // blocks on the compressed edge
  int32_t tab_off;     // first slot of the child table (in SkvSlot units)
  int32_t tab_cap;     // slots (power of two), 0 = leaf
};
struct SkvSlot {       // 16 bytes
  uint32_t hash_lo, hash_hi;
  int32_t child;       // node index, -1 = empty, -2 = removed (probing goes on)
  int32_t pad;
};
#define SKV_CTR_STRIDE 8  // uint32 per block: [0] hit_cur, [1..4] tenant bitmap, [5] hit_pre, [6] u_pre, [7] predicate streak

struct SkvTreeDev {
  const int32_t* tok;     // [n_blocks][16]
  const int32_t* page;    // [n_blocks]   address vector
  int32_t* meta;          // [n_blocks]   bit31 = private_tag, bits 0..30 = creator_id (demotion sets bit31)
  const int32_t* canon;   // [n_blocks]   input block id that created the entry
  const int32_t* flat_of; // [n_in_blocks] flat index of the entry an input block created, -1 if none
  uint32_t* ctr;          // [n_blocks][SKV_CTR_STRIDE]
  uint32_t* epoch;        // [n_blocks]   epoch counter value at the block's last access
  uint32_t* limits;       // [1] SKV_LIMIT_* bits of the limits the branching lookup has run into since the last read
  const SkvNode* nodes;   // [n_nodes+1]
  const SkvSlot* slots;
  int32_t n_blocks, n_nodes, n_tenants, n_pages;  // n_blocks: block records in use, evicted ones (canon < 0) included
  uint32_t cur_epoch;     // stamped on every block a lookup matches
};

struct SkvHostMirror;  // host copy of the structure, kept for insertions
struct skv_tree {
  SkvTreeDev dev;
  int64_t n_in_blocks;
  int device;
  SkvHostMirror* host;
  int has_copies;  // some position holds several children with the same first block: lookups must branch
};

// ---- block hash (host builds the tables, device probes them) -------------------------------
SKV_HD inline uint64_t skv_mix_tok(uint32_t tok, uint32_t i) {
  uint64_t x = (uint64_t)tok + 0x9E3779B97F4A7C15ull * (uint64_t)(i + 1);
  x ^= x >> 32; x *= 0xD6E8FEB86659FD93ull;
  x ^= x >> 32; x *= 0xD6E8FEB86659FD93ull;
  x ^= x >> 32;
  return x;
}
SKV_HD inline uint64_t skv_hash_fin(uint64_t s) {
  s ^= s >> 29; s *= 0xBF58476D1CE4E5B9ull;
  s ^= s >> 32;
  return s;
}
inline uint64_t skv_hash_block_host(const int32_t* tok) {
  uint64_t s = 0;
  for (uint32_t i = 0; i < 16; ++i) s += skv_mix_tok((uint32_t)tok[i], i);
  return skv_hash_fin(s);
}

// ---- error plumbing ---------------------------------------------------------------------------
void skv_set_hip_error(int e);
#define SKV_HIP(call)                          \
  do {                                         \
    hipError_t e_ = (call);                    \
    if (e_ != hipSuccess) {                    \
      skv_set_hip_error((int)e_);              \
      return SKV_EHIP;                         \
    }                                          \
  } while (0)

static inline size_t skv_align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Softmax scale of an attention description: the caller's value when it is a positive finite number,
// otherwise 1/sqrt(head_dim) (scaled dot-product attention, SafeKV Section 2.1).
static inline float skv_softmax_scale(const skv_attn_desc* d) {
  const float s = d->scale;
  if (s > 0.f && s < 3.0e38f) return s;
  return 1.0f / sqrtf((float)d->head_dim);
}

#endif
