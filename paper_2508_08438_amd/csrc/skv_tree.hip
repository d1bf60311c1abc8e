// Index construction (host) and counter read-back / reset kernels.
//
// SafeKV Section 4.3.1 (Insert: blocks are appended along the radix-tree path, each entry
// recording private_tag and creator_id) and Section 4.3.2 (path compression: a chain is
// collapsed into one composite node that aggregates the KV addresses of the chain in a
// vector).  The tree is built without pointers: every distinct block-prefix gets an id
// through one hash table keyed by (parent id, 16 tokens); non-branching runs are then laid
// out contiguously and only branch points keep a child table.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "skv_internal.h"

static thread_local int g_last_hip_error = 0;
void skv_set_hip_error(int e) { g_last_hip_error = e; }

extern "C" int skv_last_hip_error(void) { return g_last_hip_error; }

extern "C" const char* skv_strerror(int code) {
  switch (code) {
    case SKV_OK: return "ok";
    case SKV_EINVAL: return "invalid argument";
    case SKV_ENOMEM: return "caller-provided device buffer too small";
    case SKV_ERANGE: return "value exceeds a built-in limit";
    case SKV_EHIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

namespace {

constexpr int64_t kMaxBlocks = 0x7fffffff / 32;

struct Layout {  // byte offsets inside the slab
  size_t tok, page, meta, canon, flat_of, ctr, epoch, status, nodes, slots, total;
};

// Every array is sized for `cap` blocks: the entries the build creates plus room for later insertions.
// A node holds at least one block, so cap + 1 node records always suffice; child tables are kept at most
// half full and an outgrown table is left behind in the arena, which 8 slots per block cover.
size_t slots_for(size_t cap) { return 8 * cap + 8; }

Layout make_layout(size_t n_blocks, size_t n_in_blocks, size_t n_nodes_incl_root, size_t n_slots) {
  Layout l;
  size_t o = 0;
  l.tok = o;   o = skv_align256(o + n_blocks * 16 * sizeof(int32_t));
  l.page = o;  o = skv_align256(o + n_blocks * sizeof(int32_t));
  l.meta = o;  o = skv_align256(o + n_blocks * sizeof(int32_t));
  l.canon = o; o = skv_align256(o + n_blocks * sizeof(int32_t));
  l.flat_of = o; o = skv_align256(o + (n_in_blocks ? n_in_blocks : 1) * sizeof(int32_t));
  l.nodes = o; o = skv_align256(o + n_nodes_incl_root * sizeof(SkvNode));
  l.slots = o; o = skv_align256(o + (n_slots ? n_slots : 1) * sizeof(SkvSlot));
  l.ctr = o;   o = skv_align256(o + n_blocks * SKV_CTR_STRIDE * sizeof(uint32_t));
  l.epoch = o; o = skv_align256(o + (n_blocks ? n_blocks : 1) * sizeof(uint32_t));
  l.status = o; o = skv_align256(o + 64 * sizeof(uint32_t));   // word 0: limits the branching lookup ran into
  l.total = o;
  return l;
}

}  // namespace

// Host copy of the structure (not of the visibility bits or counters, which kernels change): what an
// insertion has to read and extend.
struct SkvHostMirror {
  Layout L;
  char* base = nullptr;               // the slab
  int64_t cap_blocks = 0;
  size_t slots_used = 0;
  std::vector<SkvNode> nodes;         // [n_nodes + 1]
  std::vector<int32_t> kids;          // children per node
  std::vector<int32_t> filled;        // table slots that are not empty (children + removed entries)
  std::vector<int32_t> parent;        // parent node of every node (root: -1)
  std::vector<SkvSlot> slots;         // the arena up to slots_used
  std::vector<int32_t> tok;           // [n_blocks][16], flat order
  std::vector<int32_t> canon, page;   // [n_blocks] input block id (-1 once evicted), page id
  std::vector<int32_t> flat_of;       // [n_in_blocks]
  std::vector<int32_t> node_of;       // [n_blocks] node that holds each block record (path ends name records)
  std::vector<uint8_t> page_used;     // [n_pages]
  int64_t live_blocks = 0;
  // Visibility words as the host last knew them.  Kernels change them (promotion, the safeguard's demotion), so
  // every call that enqueues such a kernel marks the copy stale and the next reader fetches it again.
  std::vector<int32_t> vis;           // [n_blocks]
  bool vis_stale = false;
};

namespace {

int check_desc(const skv_tree_desc* d, int64_t* n_in_blocks) {
  if (!d || !d->seq_off) return SKV_EINVAL;
  if (d->block_tokens != SKV_BLOCK_TOKENS) return SKV_EINVAL;
  if (d->n_tenants < 1 || d->n_tenants > SKV_MAX_TENANTS) return SKV_ERANGE;
  if (d->n_pages < 1 || d->n_seq < 0) return SKV_EINVAL;
  if (d->seq_off[0] != 0) return SKV_EINVAL;
  for (int64_t s = 0; s < d->n_seq; ++s) {
    if (d->seq_off[s + 1] < d->seq_off[s] || d->seq_off[s + 1] % SKV_BLOCK_TOKENS) return SKV_EINVAL;
  }
  int64_t nib = d->seq_off[d->n_seq] / SKV_BLOCK_TOKENS;
  if (nib > kMaxBlocks) return SKV_ERANGE;
  if (nib > 0 && (!d->tokens || !d->blk_sensitive || !d->blk_owner || !d->blk_page)) return SKV_EINVAL;
  *n_in_blocks = nib;
  return SKV_OK;
}

Layout layout_for(size_t cap) { return make_layout(cap, cap, cap + 1, slots_for(cap)); }

uint32_t next_pow2(uint32_t x) {
  uint32_t p = 1;
  while (p < x) p <<= 1;
  return p;
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = v;
}

__global__ void counters_scatter_kernel(SkvTreeDev t, uint32_t* hit, uint32_t* ucnt) {
  for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < t.n_blocks; b += gridDim.x * blockDim.x) {
    const uint32_t* c = t.ctr + (size_t)b * SKV_CTR_STRIDE;
    int id = t.canon[b];
    if (id < 0) continue;  // evicted
    hit[id] = c[0];
    ucnt[id] = __popc(c[1]) + __popc(c[2]) + __popc(c[3]) + __popc(c[4]);
  }
}

__global__ void counters_clear_window_kernel(SkvTreeDev t) {
  for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < t.n_blocks; b += gridDim.x * blockDim.x) {
    uint32_t* c = t.ctr + (size_t)b * SKV_CTR_STRIDE;
    c[0] = 0; c[1] = 0; c[2] = 0; c[3] = 0; c[4] = 0;
  }
}

// Safeguard step (SafeKV Section 4.2.2, Section 6): one thread per block; a streaming pass over the
// counter records (32 B read + 32 B written per block) and the metadata word.
__global__ void window_roll_kernel(SkvTreeDev t, skv_rdr_policy pol, int32_t* n_demoted) {
  for (int b0 = blockIdx.x * blockDim.x; b0 < t.n_blocks; b0 += gridDim.x * blockDim.x) {
    const int b = b0 + threadIdx.x;
    bool demote = false;
    if (b < t.n_blocks && t.canon[b] >= 0) {  // evicted records are skipped
      uint4* rec = (uint4*)(t.ctr + (size_t)b * SKV_CTR_STRIDE);
      const uint4 lo = rec[0], hi = rec[1];  // {hit, bm0, bm1, bm2}, {bm3, hit_pre, u_pre, streak}
      const uint32_t h = lo.x;
      const uint32_t u = __popc(lo.y) + __popc(lo.z) + __popc(lo.w) + __popc(hi.x);
      bool pred = false;
      if (h > 0 && h >= pol.min_hits) {
        const unsigned long long lhs = (unsigned long long)u * pol.tau_den, rhs = (unsigned long long)pol.tau_num * h;
        pred = pol.direction == 0 ? lhs < rhs : (lhs > rhs && hi.z <= pol.u_pre_max);
      }
      uint32_t streak = pred ? hi.w + 1 : 0;
      const int m = t.meta[b];
      if (m >= 0 && streak >= pol.n_consec) {  // shareable (bit 31 clear) and the predicate held long enough
        t.meta[b] = m | (int)0x80000000;
        streak = 0;
        demote = true;
      }
      rec[0] = make_uint4(0u, 0u, 0u, 0u);
      rec[1] = make_uint4(0u, h, u, streak);
    }
    if (n_demoted) {
      const unsigned long long mask = __ballot(demote);
      if (mask && (threadIdx.x & 63) == 0) atomicAdd(n_demoted, (int)__popcll(mask));
    }
  }
}

__global__ void block_state_scatter_kernel(SkvTreeDev t, uint8_t* priv, uint32_t* hit_pre, uint32_t* u_pre) {
  for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < t.n_blocks; b += gridDim.x * blockDim.x) {
    const uint32_t* c = t.ctr + (size_t)b * SKV_CTR_STRIDE;
    const int id = t.canon[b];
    if (id < 0) continue;  // evicted
    if (priv) priv[id] = t.meta[b] < 0 ? 1 : 0;
    if (hit_pre) hit_pre[id] = c[5];
    if (u_pre) u_pre[id] = c[6];
  }
}

__global__ void epoch_scatter_kernel(SkvTreeDev t, uint32_t* epoch) {
  for (int b = blockIdx.x * blockDim.x + threadIdx.x; b < t.n_blocks; b += gridDim.x * blockDim.x) {
    const int id = t.canon[b];
    if (id >= 0) epoch[id] = t.epoch[b];
  }
}

__global__ void promote_kernel(SkvTreeDev t, int64_t n_in_blocks, const int32_t* ids, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    const int id = ids[i];
    if (id < 0 || id >= n_in_blocks) continue;
    const int f = t.flat_of[id];
    if (f >= 0) atomicAnd((unsigned int*)&t.meta[f], 0x7fffffffu);  // the visibility bit flips atomically
  }
}

__global__ void fill_u8_kernel(uint8_t* p, size_t n, uint8_t v) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

int grid_for(size_t n, int block) {
  size_t g = (n + block - 1) / block;
  if (g < 1) g = 1;
  if (g > 4096) g = 4096;
  return (int)g;
}

}  // namespace

extern "C" int skv_tree_build_size(const skv_tree_desc* desc, size_t* device_bytes) {
  int64_t nib = 0;
  int rc = check_desc(desc, &nib);
  if (rc) return rc;
  if (!device_bytes) return SKV_EINVAL;
  *device_bytes = layout_for((size_t)nib).total;
  return SKV_OK;
}

extern "C" int skv_tree_size_for_capacity(int64_t block_capacity, size_t* device_bytes) {
  if (block_capacity < 0 || !device_bytes) return SKV_EINVAL;
  if (block_capacity > kMaxBlocks) return SKV_ERANGE;
  *device_bytes = layout_for((size_t)block_capacity).total;
  return SKV_OK;
}

extern "C" int skv_tree_build(const skv_tree_desc* d, void* d_slab, size_t bytes, void* stream,
                              skv_tree** out) {
  int64_t nib64 = 0;
  int rc = check_desc(d, &nib64);
  if (rc) return rc;
  if (!out || !d_slab || ((uintptr_t)d_slab & 255)) return SKV_EINVAL;
  const int32_t nib = (int32_t)nib64;
  for (int32_t b = 0; b < nib; ++b) {
    if (d->blk_owner[b] < 0 || d->blk_owner[b] >= d->n_tenants) return SKV_EINVAL;
    if (d->blk_page[b] < 0 || d->blk_page[b] >= d->n_pages) return SKV_EINVAL;
  }

  // 1. one id per distinct block-prefix: hash table over (parent id, 16 tokens), first wins
  std::vector<int32_t> parent, src, n_child, only_child;
  std::vector<uint64_t> bhash;  // hash of the block's own 16 tokens
  parent.reserve(nib); src.reserve(nib); n_child.reserve(nib); only_child.reserve(nib); bhash.reserve(nib);
  const uint32_t cap = next_pow2((uint32_t)(2 * (size_t)nib + 2));
  std::vector<int32_t> table(cap, -1);
  for (int64_t s = 0; s < d->n_seq; ++s) {
    int32_t par = -1;
    for (int64_t b = d->seq_off[s] / 16; b < d->seq_off[s + 1] / 16; ++b) {
      const int32_t* tk = d->tokens + b * 16;
      const uint64_t hb = skv_hash_block_host(tk);
      uint32_t slot = (uint32_t)skv_hash_fin(hb + 0x632BE59BD9B4E019ull * (uint64_t)(uint32_t)(par + 1)) & (cap - 1);
      int32_t id;
      for (;;) {
        id = table[slot];
        if (id < 0) break;
        if (parent[id] == par && bhash[id] == hb && !memcmp(d->tokens + (size_t)src[id] * 16, tk, 64)) break;
        slot = (slot + 1) & (cap - 1);
      }
      if (id < 0) {
        id = (int32_t)parent.size();
        table[slot] = id;
        parent.push_back(par); src.push_back((int32_t)b); n_child.push_back(0);
        only_child.push_back(-1); bhash.push_back(hb);
        if (par >= 0) { n_child[par]++; only_child[par] = id; }
      }
      par = id;
    }
  }
  const int32_t n_blocks = (int32_t)parent.size();
  {  // one KV page may back only one cached block
    std::vector<uint8_t> used((size_t)d->n_pages, 0);
    for (int32_t b = 0; b < n_blocks; ++b) {
      int32_t p = d->blk_page[src[b]];
      if (used[p]) return SKV_EINVAL;
      used[p] = 1;
    }
  }

  // 2. nodes = maximal non-branching runs; flat order = node after node
  std::vector<int32_t> flat(n_blocks), node_of(n_blocks);
  std::vector<SkvNode> nodes(1, SkvNode{0, 0, 0, 0});
  std::vector<int32_t> head_of_node(1, -1);
  int32_t next_flat = 0;
  for (int32_t b = 0; b < n_blocks; ++b) {
    const bool head = parent[b] < 0 || n_child[parent[b]] != 1;
    if (!head) continue;
    SkvNode nd{next_flat, 0, 0, 0};
    const int32_t id = (int32_t)nodes.size();
    for (int32_t c = b;; c = only_child[c]) {
      flat[c] = next_flat++;
      node_of[c] = id;
      nd.n_blocks++;
      if (n_child[c] != 1) break;
    }
    nodes.push_back(nd);
    head_of_node.push_back(b);
  }
  const int32_t n_nodes = (int32_t)nodes.size() - 1;

  // 3. child tables at branch points
  std::vector<int32_t> kids(n_nodes + 1, 0);
  for (int32_t n = 1; n <= n_nodes; ++n) {
    int32_t p = parent[head_of_node[n]];
    kids[p < 0 ? 0 : node_of[p]]++;
  }
  size_t n_slots = 0;
  for (int32_t n = 0; n <= n_nodes; ++n) {
    nodes[n].tab_off = (int32_t)n_slots;
    nodes[n].tab_cap = kids[n] ? (int32_t)next_pow2(2u * (uint32_t)kids[n]) : 0;
    n_slots += (size_t)nodes[n].tab_cap;
  }
  if (n_slots > 0x7fffffff) return SKV_ERANGE;
  std::vector<SkvSlot> slots(n_slots ? n_slots : 1, SkvSlot{0, 0, -1, 0});
  for (int32_t n = 1; n <= n_nodes; ++n) {
    const int32_t hb = head_of_node[n];
    const SkvNode& pn = nodes[parent[hb] < 0 ? 0 : node_of[parent[hb]]];
    const uint64_t h = bhash[hb];
    uint32_t s = (uint32_t)h & (uint32_t)(pn.tab_cap - 1);
    while (slots[pn.tab_off + s].child >= 0) s = (s + 1) & (uint32_t)(pn.tab_cap - 1);
    slots[pn.tab_off + s] = SkvSlot{(uint32_t)h, (uint32_t)(h >> 32), n, 0};
  }

  // 4. stage and upload.  The slab's size fixes the capacity: the largest block count whose layout fits.
  if (layout_for((size_t)nib).total > bytes) return SKV_ENOMEM;
  int64_t cap_blocks = nib;
  for (int64_t lo = nib, hi = kMaxBlocks; lo <= hi;) {
    const int64_t mid = lo + (hi - lo) / 2;
    if (layout_for((size_t)mid).total <= bytes) { cap_blocks = mid; lo = mid + 1; } else { hi = mid - 1; }
  }
  const Layout L = layout_for((size_t)cap_blocks);
  if (n_slots > slots_for((size_t)cap_blocks)) return SKV_ENOMEM;
  std::vector<char> host(L.slots + (n_slots ? n_slots : 1) * sizeof(SkvSlot));  // everything up to the used slots
  int32_t* h_tok = (int32_t*)(host.data() + L.tok);
  int32_t* h_page = (int32_t*)(host.data() + L.page);
  int32_t* h_meta = (int32_t*)(host.data() + L.meta);
  int32_t* h_canon = (int32_t*)(host.data() + L.canon);
  int32_t* h_flat_of = (int32_t*)(host.data() + L.flat_of);
  for (int32_t b = 0; b < nib; ++b) h_flat_of[b] = -1;
  for (int32_t b = 0; b < n_blocks; ++b) {
    const int32_t f = flat[b], in = src[b];
    memcpy(h_tok + (size_t)f * 16, d->tokens + (size_t)in * 16, 64);
    h_page[f] = d->blk_page[in];
    h_meta[f] = (d->blk_sensitive[in] ? (int32_t)0x80000000 : 0) | d->blk_owner[in];
    h_canon[f] = in;
    h_flat_of[in] = f;
  }
  memcpy(host.data() + L.nodes, nodes.data(), nodes.size() * sizeof(SkvNode));
  memcpy(host.data() + L.slots, slots.data(), slots.size() * sizeof(SkvSlot));

  skv_tree* t = new (std::nothrow) skv_tree();
  if (!t) return SKV_EINVAL;
  char* base = (char*)d_slab;
  SkvHostMirror* m = new (std::nothrow) SkvHostMirror();
  if (!m) { delete t; return SKV_EINVAL; }
  t->host = m;
  t->has_copies = 0;
  m->L = L;
  m->base = base;
  m->cap_blocks = cap_blocks;
  m->slots_used = n_slots;
  m->nodes = nodes;
  m->kids = kids;
  m->filled = kids;
  m->parent.assign(nodes.size(), -1);
  for (int32_t n = 1; n <= n_nodes; ++n) {
    const int32_t pb = parent[head_of_node[n]];
    m->parent[n] = pb < 0 ? 0 : node_of[pb];
  }
  m->canon.assign(h_canon, h_canon + n_blocks);
  m->page.assign(h_page, h_page + n_blocks);
  m->vis.assign(h_meta, h_meta + n_blocks);
  m->node_of.assign((size_t)n_blocks, 0);
  for (int32_t n = 1; n <= n_nodes; ++n)
    for (int32_t k = 0; k < nodes[n].n_blocks; ++k) m->node_of[(size_t)nodes[n].first + k] = n;
  m->flat_of.assign(h_flat_of, h_flat_of + nib);
  m->live_blocks = n_blocks;
  m->slots.assign(slots.begin(), slots.begin() + n_slots);
  m->tok.assign(h_tok, h_tok + (size_t)n_blocks * 16);
  m->page_used.assign((size_t)d->n_pages, 0);
  for (int32_t b = 0; b < n_blocks; ++b) m->page_used[h_page[b]] = 1;
  t->dev.tok = (const int32_t*)(base + L.tok);
  t->dev.page = (const int32_t*)(base + L.page);
  t->dev.meta = (int32_t*)(base + L.meta);
  t->dev.canon = (const int32_t*)(base + L.canon);
  t->dev.flat_of = (const int32_t*)(base + L.flat_of);
  t->dev.ctr = (uint32_t*)(base + L.ctr);
  t->dev.epoch = (uint32_t*)(base + L.epoch);
  t->dev.limits = (uint32_t*)(base + L.status);
  t->dev.cur_epoch = 0;
  t->dev.nodes = (const SkvNode*)(base + L.nodes);
  t->dev.slots = (const SkvSlot*)(base + L.slots);
  t->dev.n_blocks = n_blocks;
  t->dev.n_nodes = n_nodes;
  t->dev.n_tenants = d->n_tenants;
  t->dev.n_pages = d->n_pages;
  t->n_in_blocks = nib;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = hipGetDevice(&t->device);
  if (e == hipSuccess) e = hipMemcpyAsync(base, host.data(), host.size(), hipMemcpyHostToDevice, st);
  if (e == hipSuccess && cap_blocks) {  // counters of the whole capacity: inserted blocks start from zero
    size_t n = (size_t)cap_blocks * SKV_CTR_STRIDE;
    fill_u32_kernel<<<grid_for(n, 256), 256, 0, st>>>(t->dev.ctr, n, 0u);
    fill_u32_kernel<<<grid_for((size_t)cap_blocks, 256), 256, 0, st>>>(t->dev.epoch, (size_t)cap_blocks, 0u);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    fill_u32_kernel<<<1, 64, 0, st>>>(t->dev.limits, 64, 0u);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) {
    skv_set_hip_error((int)e);
    delete m;
    delete t;
    return SKV_EHIP;
  }
  *out = t;
  return SKV_OK;
}

// ---- insertion after prefill (Section 4.3.1 Insert; Section 4.1 and Section 6: new blocks are private by default) ----
namespace {

struct Inserter {
  skv_tree* t;
  SkvHostMirror* m;
  int64_t n_blocks, n_in;            // running totals
  std::vector<int32_t> page, meta;   // per appended block
  size_t node_lo, node_hi, slot_lo, slot_hi;  // dirty spans of records that existed before [lo, hi)
  bool full = false;

  void touch_node(size_t i) { node_lo = std::min(node_lo, i); node_hi = std::max(node_hi, i + 1); }
  void touch_slot(size_t i) { slot_lo = std::min(slot_lo, i); slot_hi = std::max(slot_hi, i + 1); }

  int32_t find_child(int32_t node, const int32_t* blk, uint64_t h) const {
    const SkvNode& n = m->nodes[node];
    if (!n.tab_cap) return -1;
    for (uint32_t s = (uint32_t)h & (uint32_t)(n.tab_cap - 1);; s = (s + 1) & (uint32_t)(n.tab_cap - 1)) {
      const SkvSlot& sl = m->slots[(size_t)n.tab_off + s];
      if (sl.child == -1) return -1;
      if (sl.child >= 0 && sl.hash_lo == (uint32_t)h && sl.hash_hi == (uint32_t)(h >> 32) &&
          !memcmp(&m->tok[(size_t)m->nodes[sl.child].first * 16], blk, 64))
        return sl.child;
    }
  }
  void put(int32_t node, uint64_t h, int32_t child) {  // into the first empty or removed slot of the probe sequence
    const SkvNode& n = m->nodes[node];
    uint32_t s = (uint32_t)h & (uint32_t)(n.tab_cap - 1);
    while (m->slots[(size_t)n.tab_off + s].child >= 0) s = (s + 1) & (uint32_t)(n.tab_cap - 1);
    if (m->slots[(size_t)n.tab_off + s].child == -1) m->filled[node]++;
    m->slots[(size_t)n.tab_off + s] = SkvSlot{(uint32_t)h, (uint32_t)(h >> 32), child, 0};
    touch_slot((size_t)n.tab_off + s);
  }
  // Adds a child; a table that would become more than half full moves to a fresh one of twice the size.
  bool add_child(int32_t node, uint64_t h, int32_t child) {
    SkvNode& n = m->nodes[node];
    const int32_t kids = m->kids[node] + 1;
    if (2 * (m->filled[node] + 1) > n.tab_cap) {  // removed entries count: a probe must always reach an empty slot
      const int32_t cap = (int32_t)next_pow2((uint32_t)(2 * kids) < 4u ? 4u : (uint32_t)(2 * kids));
      if (m->slots_used + (size_t)cap > slots_for((size_t)m->cap_blocks)) return false;
      const SkvNode old = n;
      n.tab_off = (int32_t)m->slots_used;
      n.tab_cap = cap;
      m->slots_used += (size_t)cap;
      m->slots.resize(m->slots_used, SkvSlot{0, 0, -1, 0});
      touch_slot((size_t)n.tab_off);
      touch_slot(m->slots_used - 1);
      m->filled[node] = 0;
      for (int32_t i = 0; i < old.tab_cap; ++i) {
        const SkvSlot sl = m->slots[(size_t)old.tab_off + i];
        if (sl.child >= 0) put(node, ((uint64_t)sl.hash_hi << 32) | sl.hash_lo, sl.child);
      }
      touch_node((size_t)node);
    }
    put(node, h, child);
    m->kids[node] = kids;
    return true;
  }
  // ---- private copies (Section 4.1): where the requester's own longest visible path ends ----
  // Several children of a node may start with the same block (one copy per tenant that could not see the others),
  // so the path is not unique and has to be searched: a stack of open positions, each with the copies that match
  // the request's next block ordered by the input id of their first block (the oldest copy is tried first).  A copy
  // is followed for as many blocks as match and are visible; if that covers the whole node the position below it
  // is opened, otherwise the path ends inside the node.  The first end that reaches the greatest depth is kept.
  struct PathEnd { int32_t node = 0, used = 0; int64_t depth = -1; };
  struct OpenPos {
    int32_t node;
    int64_t depth;
    std::vector<std::pair<int32_t, int32_t>> copies;  // (input id of the copy's first block, child node)
    size_t next = 0;
    bool extended = false;                             // some copy took the path further than this node
  };
  void matching_copies(int32_t node, const int32_t* blk, std::vector<std::pair<int32_t, int32_t>>& out) const {
    const SkvNode& n = m->nodes[node];
    if (!n.tab_cap) return;
    const uint64_t h = skv_hash_block_host(blk);
    const uint32_t mask = (uint32_t)(n.tab_cap - 1);
    for (uint32_t s = (uint32_t)h & mask; m->slots[(size_t)n.tab_off + s].child != -1; s = (s + 1) & mask) {
      const SkvSlot& sl = m->slots[(size_t)n.tab_off + s];
      if (sl.child < 0 || sl.hash_lo != (uint32_t)h || sl.hash_hi != (uint32_t)(h >> 32)) continue;
      const int32_t f = m->nodes[sl.child].first;
      if (!memcmp(&m->tok[(size_t)f * 16], blk, 64)) out.push_back({m->canon[f], sl.child});
    }
    std::sort(out.begin(), out.end());
  }
  int32_t visible_run(const SkvNode& c, const int32_t* x, int64_t room, int32_t tenant) const {
    const int64_t lim = std::min<int64_t>(c.n_blocks, room);
    int64_t k = 0;
    for (; k < lim; ++k) {
      const int32_t word = m->vis[(size_t)c.first + k];
      if (word < 0 && (word & 0x7fffffff) != tenant) break;   // private to somebody else
      if (memcmp(&m->tok[((size_t)c.first + k) * 16], x + k * 16, 64)) break;
    }
    return (int32_t)k;
  }
  PathEnd longest_visible_path(const int32_t* x, int64_t nb, int32_t tenant) const {
    PathEnd best;
    std::vector<OpenPos> open;
    auto open_at = [&](int32_t node, int64_t depth) {
      open.push_back(OpenPos{node, depth, {}});
      if (depth < nb) matching_copies(node, x + depth * 16, open.back().copies);
    };
    auto offer = [&](int32_t node, int32_t used, int64_t depth) {
      if (depth > best.depth) best = PathEnd{node, used, depth};
    };
    open_at(0, 0);
    while (!open.empty() && best.depth < nb) {
      OpenPos& p = open.back();
      if (p.next == p.copies.size()) {          // every copy tried: a position nothing continued is an end itself
        if (!p.extended) offer(p.node, m->nodes[p.node].n_blocks, p.depth);
        open.pop_back();
        continue;
      }
      const int32_t child = p.copies[p.next++].second;
      const SkvNode c = m->nodes[child];
      const int32_t k = visible_run(c, x + p.depth * 16, nb - p.depth, tenant);
      if (k == 0) continue;
      p.extended = true;
      const int64_t below = p.depth + k;        // (p may dangle after the next push)
      if (k == c.n_blocks) open_at(child, below);
      else offer(child, k, below);
    }
    return best;
  }
  // Appends blocks [k, nb) of the request below the end of its own longest visible path.  Returns k, or -1
  // when the slab is full.
  int64_t insert_copy(const int32_t* x, int64_t nb, int32_t tenant, const int32_t* pages, int64_t k_vis, int64_t* n_new) {
    *n_new = 0;
    const PathEnd end = longest_visible_path(x, nb, tenant);
    const int64_t k = end.depth;
    if (k >= nb || k < k_vis) return k;
    const int32_t at = end.node;
    if (end.used < m->nodes[at].n_blocks) {  // the path stops inside a compressed edge: split it there
      if ((int64_t)m->nodes.size() + 2 > m->cap_blocks + 1) return -1;
      if (!split(at, end.used)) return -1;
    }
    const int64_t add = nb - k;
    if (n_blocks + add > m->cap_blocks || n_in + add > m->cap_blocks) return -1;
    if ((int64_t)m->nodes.size() + 1 > m->cap_blocks + 1) return -1;
    return append(at, x, k, nb, tenant, pages, k_vis, n_new) ? k : -1;
  }
  // The same with the end of the requester's path given (the record of its last matched block, -1 for none; found by
  // the lookup before this batch).  What the lookup could not see are the blocks earlier requests of this batch added
  // for the same tenant; they hang below path ends the lookup did see, so the path is continued through them and
  // nothing else: a child (or the rest of a node) counts only if its blocks were created in this batch (records from
  // nb0 on) by this tenant.  Returns the index of the first new block, or -1 when the slab is full.
  int64_t insert_below(const int32_t* x, int64_t nb, int32_t tenant, const int32_t* pages, int64_t k_vis,
                       int32_t end_rec, int64_t nb0, int64_t* n_new) {
    *n_new = 0;
    int32_t node = 0, used = 0;
    if (end_rec >= 0) {
      node = m->node_of[end_rec];
      used = end_rec - m->nodes[node].first + 1;
    }
    int64_t k = k_vis;
    auto mine = [&](int32_t rec) { return rec >= nb0 && m->vis[rec] == ((int32_t)0x80000000 | tenant); };
    while (k < nb) {
      const SkvNode nd = m->nodes[node];
      if (used < nd.n_blocks) {              // inside a node: only this batch's own blocks continue the path
        const int32_t rec = nd.first + used;
        if (!mine(rec) || memcmp(&m->tok[(size_t)rec * 16], x + k * 16, 64)) break;
        ++used;
        ++k;
        continue;
      }
      int32_t next = -1;
      if (nd.tab_cap) {
        const uint64_t h = skv_hash_block_host(x + k * 16);
        const uint32_t mask = (uint32_t)(nd.tab_cap - 1);
        for (uint32_t q = (uint32_t)h & mask; m->slots[(size_t)nd.tab_off + q].child != -1; q = (q + 1) & mask) {
          const SkvSlot& sl = m->slots[(size_t)nd.tab_off + q];
          if (sl.child < 0 || sl.hash_lo != (uint32_t)h || sl.hash_hi != (uint32_t)(h >> 32)) continue;
          const int32_t rec = m->nodes[sl.child].first;
          if (mine(rec) && !memcmp(&m->tok[(size_t)rec * 16], x + k * 16, 64)) { next = sl.child; break; }
        }
      }
      if (next < 0) break;
      node = next;
      used = 1;
      ++k;
    }
    if (k >= nb) return k;
    if (used < m->nodes[node].n_blocks) {    // the path stops inside a compressed edge: split it there
      if ((int64_t)m->nodes.size() + 2 > m->cap_blocks + 1) return -1;
      if (!split(node, used)) return -1;
    }
    const int64_t add = nb - k;
    if (n_blocks + add > m->cap_blocks || n_in + add > m->cap_blocks) return -1;
    if ((int64_t)m->nodes.size() + 1 > m->cap_blocks + 1) return -1;
    return append(node, x, k, nb, tenant, pages, k_vis, n_new) ? k : -1;
  }
  // Cuts node c after its first j blocks: a new node takes the rest together with the child table.
  bool split(int32_t c, int64_t j) {
    const SkvNode run = m->nodes[c];
    const int32_t tail = (int32_t)m->nodes.size();
    m->nodes.push_back(SkvNode{run.first + (int32_t)j, run.n_blocks - (int32_t)j, run.tab_off, run.tab_cap});
    m->kids.push_back(m->kids[c]);
    m->filled.push_back(m->filled[c]);
    m->parent.push_back(c);
    for (int32_t q = 0; q < run.tab_cap; ++q) {  // the children move below the new node
      const int32_t gc = m->slots[(size_t)run.tab_off + q].child;
      if (gc >= 0) m->parent[gc] = tail;
    }
    for (int32_t k = (int32_t)j; k < run.n_blocks; ++k) m->node_of[(size_t)run.first + k] = tail;
    m->nodes[c].n_blocks = (int32_t)j;
    m->nodes[c].tab_off = 0;
    m->nodes[c].tab_cap = 0;
    m->kids[c] = 0;
    m->filled[c] = 0;
    touch_node((size_t)c);
    touch_node((size_t)tail);
    return add_child(c, skv_hash_block_host(&m->tok[((size_t)run.first + j) * 16]), tail);
  }
  // New node with blocks [i, nb) of the request as a child of `node`.
  bool append(int32_t node, const int32_t* x, int64_t i, int64_t nb, int32_t tenant, const int32_t* pages,
              int64_t k_vis, int64_t* n_new) {
    const int64_t add = nb - i;
    const int32_t fresh = (int32_t)m->nodes.size();
    m->nodes.push_back(SkvNode{(int32_t)n_blocks, (int32_t)add, 0, 0});
    m->kids.push_back(0);
    m->filled.push_back(0);
    m->parent.push_back(node);
    touch_node((size_t)fresh);
    if (!add_child(node, skv_hash_block_host(x + i * 16), fresh)) return false;
    m->tok.insert(m->tok.end(), x + i * 16, x + nb * 16);
    for (int64_t j = i; j < nb; ++j) {
      page.push_back(pages[j - k_vis]);
      meta.push_back((int32_t)0x80000000 | tenant);
      m->vis.push_back((int32_t)0x80000000 | tenant);
      m->node_of.push_back(fresh);
      m->page.push_back(pages[j - k_vis]);
      m->canon.push_back((int32_t)(n_in + (j - i)));
      m->flat_of.push_back((int32_t)(n_blocks + (j - i)));
      m->page_used[pages[j - k_vis]] = 1;
    }
    n_blocks += add;
    n_in += add;
    *n_new = add;
    return true;
  }
  // One request: blocks [k_exist, nb) are appended as one node below the point where the path ends.
  // Returns k_exist, or -1 when the slab is full.
  int64_t insert(const int32_t* x, int64_t nb, int32_t tenant, const int32_t* pages, int64_t k_vis, int64_t* n_new) {
    *n_new = 0;
    int32_t node = 0;
    int64_t i = 0;
    while (i < nb) {
      const uint64_t h = skv_hash_block_host(x + i * 16);
      const int32_t c = find_child(node, x + i * 16, h);
      if (c < 0) break;
      const SkvNode run = m->nodes[c];
      int64_t j = 1;
      while (j < run.n_blocks && i + j < nb && !memcmp(&m->tok[((size_t)run.first + j) * 16], x + (i + j) * 16, 64)) ++j;
      if (j < run.n_blocks) {
        if (i + j == nb) return nb;  // the request ends inside the run: nothing new
        if (i + j < k_vis) return i + j;  // caller's matched length is not one this tree gives
        // split: the run keeps its first j blocks, a new node takes the rest together with the child table
        if ((int64_t)m->nodes.size() + 2 > m->cap_blocks + 1) return -1;
        if (!split(c, j)) return -1;
        node = c;
        i += j;
        break;
      }
      node = c;
      i += j;
    }
    if (i >= nb || i < k_vis) return i;
    const int64_t add = nb - i;
    if (n_blocks + add > m->cap_blocks || n_in + add > m->cap_blocks) return -1;
    if (!append(node, x, i, nb, tenant, pages, k_vis, n_new)) return -1;
    return i;
  }
};

}  // namespace

extern "C" int skv_tree_insert(skv_tree* t, int32_t n_req, const int32_t* req_off, const int32_t* req_tokens,
                               const int32_t* req_tenant, const int32_t* matched_len, const int32_t* new_pages,
                               int32_t max_new_blocks, int32_t private_copies, const int32_t* path_end,
                               int32_t* first_inserted, int32_t* n_inserted, void* stream) {
  if (!t || !t->host || n_req < 0 || max_new_blocks < 0) return SKV_EINVAL;
  if (n_req == 0) return SKV_OK;
  if (!req_off || !req_tenant || !matched_len || !first_inserted || !n_inserted) return SKV_EINVAL;
  if (max_new_blocks > 0 && !new_pages) return SKV_EINVAL;
  SkvHostMirror* m = t->host;
  // validate everything before anything changes
  std::vector<int32_t> have(n_req, 0);
  {
    std::vector<uint8_t> seen(m->page_used.size(), 0);
    for (int32_t r = 0; r < n_req; ++r) {
      if (req_off[r + 1] < req_off[r] || req_off[r] < 0 || matched_len[r] < 0) return SKV_EINVAL;
      if (req_off[r + 1] > req_off[r] && !req_tokens) return SKV_EINVAL;
      if (req_tenant[r] < 0 || req_tenant[r] >= t->dev.n_tenants) return SKV_EINVAL;
      int32_t h = 0;
      for (; h < max_new_blocks; ++h) {
        const int32_t pg = new_pages[(size_t)r * max_new_blocks + h];
        if (pg < 0) break;
        if (pg >= t->dev.n_pages || m->page_used[pg] || seen[pg]) return SKV_EINVAL;
        seen[pg] = 1;
      }
      have[r] = h;
      if (private_copies && path_end) {   // the record must be this request's last matched block
        const int64_t k_vis = matched_len[r] / SKV_BLOCK_TOKENS;
        const int32_t e = path_end[r];
        if (k_vis == 0 ? e != -1
                       : (e < 0 || e >= t->dev.n_blocks || m->canon[e] < 0 ||
                          k_vis * SKV_BLOCK_TOKENS > req_off[r + 1] - req_off[r] ||
                          memcmp(&m->tok[(size_t)e * 16], req_tokens + req_off[r] + (k_vis - 1) * 16, 64)))
          return SKV_EINVAL;
      }
    }
  }
  // work on the mirror; a full slab restores the snapshot and changes nothing
  const std::vector<SkvNode> nodes0 = m->nodes;
  const std::vector<int32_t> kids0 = m->kids;
  const std::vector<SkvSlot> slots0 = m->slots;
  const std::vector<uint8_t> used0 = m->page_used;
  const std::vector<int32_t> filled0 = m->filled, parent0 = m->parent, node_of0 = m->node_of;
  const size_t slots_used0 = m->slots_used, tok0 = m->tok.size(), blocks0 = m->canon.size(), in0 = m->flat_of.size();
  Inserter ins{t, m, t->dev.n_blocks, t->n_in_blocks, {}, {}, SIZE_MAX, 0, SIZE_MAX, 0};
  hipStream_t st = (hipStream_t)stream;
  // The requester's own path depends on the visibility bits.  The host's copy of them is exact unless a
  // promotion or a safeguard window has been enqueued since it was taken; only then is it fetched again.
  if (private_copies && !path_end && m->vis_stale && t->dev.n_blocks) {
    SKV_HIP(hipMemcpyAsync(m->vis.data(), t->dev.meta, (size_t)t->dev.n_blocks * 4, hipMemcpyDeviceToHost, st));
    SKV_HIP(hipStreamSynchronize(st));
    m->vis_stale = false;
  }
  bool full = false;
  for (int32_t r = 0; r < n_req && !full; ++r) {
    const int64_t k_vis = matched_len[r] / SKV_BLOCK_TOKENS;
    int64_t nb = (req_off[r + 1] - req_off[r]) / SKV_BLOCK_TOKENS;
    if (nb > k_vis + have[r]) nb = k_vis + have[r];
    int64_t n_new = 0;
    const int32_t* pages_r = new_pages + (size_t)r * max_new_blocks;
    const int32_t* x = req_tokens + req_off[r];
    const int64_t first = !private_copies ? ins.insert(x, nb, req_tenant[r], pages_r, k_vis, &n_new)
                          : path_end      ? ins.insert_below(x, nb, req_tenant[r], pages_r, k_vis, path_end[r], t->dev.n_blocks, &n_new)
                                          : ins.insert_copy(x, nb, req_tenant[r], pages_r, k_vis, &n_new);
    if (first < 0) { full = true; break; }
    first_inserted[r] = (int32_t)first;
    n_inserted[r] = (int32_t)n_new;
  }
  if (full) {
    m->nodes = nodes0; m->kids = kids0; m->slots = slots0; m->page_used = used0;
    m->filled = filled0; m->parent = parent0; m->node_of = node_of0;
    m->slots_used = slots_used0; m->tok.resize(tok0);
    m->canon.resize(blocks0); m->page.resize(blocks0); m->vis.resize(blocks0); m->flat_of.resize(in0);
    return SKV_ENOMEM;
  }
  // upload: the appended block records, then the spans of node and slot records that changed
  const int64_t nb0 = t->dev.n_blocks, nin0 = t->n_in_blocks, add = ins.n_blocks - nb0;
  char* base = m->base;
  if (private_copies && add > 0) t->has_copies = 1;
  if (add > 0) {
    std::vector<int32_t> canon((size_t)add), flat_of((size_t)add);
    for (int64_t i = 0; i < add; ++i) { canon[i] = (int32_t)(nin0 + i); flat_of[i] = (int32_t)(nb0 + i); }
    SKV_HIP(hipMemcpyAsync(base + m->L.tok + (size_t)nb0 * 64, &m->tok[(size_t)nb0 * 16], (size_t)add * 64, hipMemcpyHostToDevice, st));
    SKV_HIP(hipMemcpyAsync(base + m->L.page + (size_t)nb0 * 4, ins.page.data(), (size_t)add * 4, hipMemcpyHostToDevice, st));
    SKV_HIP(hipMemcpyAsync(base + m->L.meta + (size_t)nb0 * 4, ins.meta.data(), (size_t)add * 4, hipMemcpyHostToDevice, st));
    SKV_HIP(hipMemcpyAsync(base + m->L.canon + (size_t)nb0 * 4, canon.data(), (size_t)add * 4, hipMemcpyHostToDevice, st));
    SKV_HIP(hipMemcpyAsync(base + m->L.flat_of + (size_t)nin0 * 4, flat_of.data(), (size_t)add * 4, hipMemcpyHostToDevice, st));
    fill_u32_kernel<<<grid_for((size_t)add, 256), 256, 0, st>>>(t->dev.epoch + nb0, (size_t)add, t->dev.cur_epoch);
    SKV_HIP(hipGetLastError());
    SKV_HIP(hipStreamSynchronize(st));  // the staging vectors die with this scope
  }
  if (ins.node_hi > ins.node_lo)
    SKV_HIP(hipMemcpyAsync(base + m->L.nodes + ins.node_lo * sizeof(SkvNode), &m->nodes[ins.node_lo],
                           (ins.node_hi - ins.node_lo) * sizeof(SkvNode), hipMemcpyHostToDevice, st));
  if (ins.slot_hi > ins.slot_lo)
    SKV_HIP(hipMemcpyAsync(base + m->L.slots + ins.slot_lo * sizeof(SkvSlot), &m->slots[ins.slot_lo],
                           (ins.slot_hi - ins.slot_lo) * sizeof(SkvSlot), hipMemcpyHostToDevice, st));
  SKV_HIP(hipStreamSynchronize(st));
  t->dev.n_blocks = (int32_t)ins.n_blocks;
  t->dev.n_nodes = (int32_t)m->nodes.size() - 1;
  t->n_in_blocks = ins.n_in;
  m->live_blocks += add;
  return SKV_OK;
}

// ---- eviction (Section 4.3.1 Evict: epoch-based LRU; Section 4.3.2 progressive eviction) ----
extern "C" int skv_set_epoch(skv_tree* t, uint32_t epoch) {
  if (!t) return SKV_EINVAL;
  t->dev.cur_epoch = epoch;
  return SKV_OK;
}

extern "C" int skv_block_epochs_read(skv_tree* t, uint32_t* d_epoch, void* stream) {
  if (!t || !d_epoch) return SKV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  if (t->n_in_blocks) fill_u32_kernel<<<grid_for((size_t)t->n_in_blocks, 256), 256, 0, st>>>(d_epoch, (size_t)t->n_in_blocks, 0u);
  if (t->dev.n_blocks) epoch_scatter_kernel<<<grid_for((size_t)t->dev.n_blocks, 256), 256, 0, st>>>(t->dev, d_epoch);
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_evict(skv_tree* t, int64_t n_want, const int32_t* protect_ids, int64_t n_protect,
                         int32_t* evicted_ids, int32_t* evicted_pages, int64_t* n_evicted, void* stream) {
  if (!t || !t->host || n_want < 0 || n_protect < 0 || !n_evicted) return SKV_EINVAL;
  if (n_protect > 0 && !protect_ids) return SKV_EINVAL;
  if (n_want > 0 && (!evicted_ids || !evicted_pages)) return SKV_EINVAL;
  *n_evicted = 0;
  SkvHostMirror* m = t->host;
  const int64_t nb = t->dev.n_blocks;
  if (n_want == 0 || nb == 0) return SKV_OK;
  hipStream_t st = (hipStream_t)stream;
  std::vector<uint32_t> epoch((size_t)nb);
  SKV_HIP(hipMemcpyAsync(epoch.data(), t->dev.epoch, (size_t)nb * 4, hipMemcpyDeviceToHost, st));
  SKV_HIP(hipStreamSynchronize(st));
  std::vector<uint8_t> prot((size_t)t->n_in_blocks, 0);
  for (int64_t i = 0; i < n_protect; ++i)
    if (protect_ids[i] >= 0 && protect_ids[i] < t->n_in_blocks) prot[protect_ids[i]] = 1;
  // candidates: the last block of every childless node, oldest (epoch, block id) first
  struct Cand { uint32_t epoch; int32_t id, node; };
  auto later = [](const Cand& a, const Cand& b) { return a.epoch != b.epoch ? a.epoch > b.epoch : a.id > b.id; };
  std::vector<Cand> heap;
  auto push_tail = [&](int32_t n) {
    const SkvNode& nd = m->nodes[n];
    const int32_t f = nd.first + nd.n_blocks - 1;
    heap.push_back(Cand{epoch[f], m->canon[f], n});
    std::push_heap(heap.begin(), heap.end(), later);
  };
  for (int32_t n = 1; n < (int32_t)m->nodes.size(); ++n)
    if (m->kids[n] == 0 && m->nodes[n].n_blocks > 0) push_tail(n);
  size_t node_lo = SIZE_MAX, node_hi = 0, slot_lo = SIZE_MAX, slot_hi = 0, blk_lo = SIZE_MAX, blk_hi = 0, id_lo = SIZE_MAX, id_hi = 0;
  int64_t done = 0;
  while (done < n_want && !heap.empty()) {
    std::pop_heap(heap.begin(), heap.end(), later);
    const Cand c = heap.back();
    heap.pop_back();
    if (prot[c.id]) continue;  // in use: this node keeps its tail, and with it everything above
    SkvNode& nd = m->nodes[c.node];
    const int32_t f = nd.first + nd.n_blocks - 1;
    evicted_ids[done] = c.id;
    evicted_pages[done] = m->page[f];
    ++done;
    m->page_used[m->page[f]] = 0;
    m->canon[f] = -1;
    m->flat_of[c.id] = -1;
    blk_lo = std::min(blk_lo, (size_t)f); blk_hi = std::max(blk_hi, (size_t)f + 1);
    id_lo = std::min(id_lo, (size_t)c.id); id_hi = std::max(id_hi, (size_t)c.id + 1);
    nd.n_blocks--;
    node_lo = std::min(node_lo, (size_t)c.node); node_hi = std::max(node_hi, (size_t)c.node + 1);
    if (nd.n_blocks > 0) { push_tail(c.node); continue; }
    // the node is gone: its entry in the parent's table becomes a removed slot
    const int32_t p = m->parent[c.node];
    const SkvNode& pn = m->nodes[p];
    for (int32_t q = 0; q < pn.tab_cap; ++q) {
      SkvSlot& sl = m->slots[(size_t)pn.tab_off + q];
      if (sl.child == c.node) {
        sl.child = -2;
        slot_lo = std::min(slot_lo, (size_t)pn.tab_off + q); slot_hi = std::max(slot_hi, (size_t)pn.tab_off + q + 1);
        break;
      }
    }
    m->kids[p]--;
    if (m->kids[p] == 0 && p != 0 && pn.n_blocks > 0) push_tail(p);
  }
  *n_evicted = done;
  m->live_blocks -= done;
  if (!done) return SKV_OK;
  char* base = m->base;
  SKV_HIP(hipMemcpyAsync(base + m->L.canon + blk_lo * 4, &m->canon[blk_lo], (blk_hi - blk_lo) * 4, hipMemcpyHostToDevice, st));
  SKV_HIP(hipMemcpyAsync(base + m->L.flat_of + id_lo * 4, &m->flat_of[id_lo], (id_hi - id_lo) * 4, hipMemcpyHostToDevice, st));
  SKV_HIP(hipMemcpyAsync(base + m->L.nodes + node_lo * sizeof(SkvNode), &m->nodes[node_lo],
                         (node_hi - node_lo) * sizeof(SkvNode), hipMemcpyHostToDevice, st));
  if (slot_hi > slot_lo)
    SKV_HIP(hipMemcpyAsync(base + m->L.slots + slot_lo * sizeof(SkvSlot), &m->slots[slot_lo],
                           (slot_hi - slot_lo) * sizeof(SkvSlot), hipMemcpyHostToDevice, st));
  SKV_HIP(hipStreamSynchronize(st));
  return SKV_OK;
}

// ---- reclaiming record space (Section 4.3.2 Progressive Eviction: a chain's address vector shrinks as its entries
// are released and the chain itself goes once the vector is empty) ----
// Evictions shorten node runs and unlink emptied nodes, insertions abandon outgrown child tables and split runs; the
// records they leave behind stay in the slab.  Compaction lays the live structure out afresh: nodes in depth-first
// order with their blocks contiguous, child tables sized for the children they have, input block ids renumbered
// densely in their old order (so "older copy" and eviction ties still compare the same way).  The per-block state
// the kernels own (visibility bits, counters, epochs) is read back, permuted with the records and written again.
extern "C" int skv_tree_compact(skv_tree* t, int32_t* id_map, int64_t* n_in_blocks_after, void* stream) {
  if (!t || !t->host) return SKV_EINVAL;
  SkvHostMirror* m = t->host;
  hipStream_t st = (hipStream_t)stream;
  const int64_t nb_old = t->dev.n_blocks, nin_old = t->n_in_blocks;
  if (nin_old > 0 && !id_map) return SKV_EINVAL;
  std::vector<int32_t> meta((size_t)nb_old);
  std::vector<uint32_t> ctr((size_t)nb_old * SKV_CTR_STRIDE), epoch((size_t)nb_old);
  if (nb_old) {
    SKV_HIP(hipMemcpyAsync(meta.data(), t->dev.meta, (size_t)nb_old * 4, hipMemcpyDeviceToHost, st));
    SKV_HIP(hipMemcpyAsync(ctr.data(), t->dev.ctr, (size_t)nb_old * SKV_CTR_STRIDE * 4, hipMemcpyDeviceToHost, st));
    SKV_HIP(hipMemcpyAsync(epoch.data(), t->dev.epoch, (size_t)nb_old * 4, hipMemcpyDeviceToHost, st));
    SKV_HIP(hipStreamSynchronize(st));
  }
  // dense input ids, old order kept
  std::vector<int32_t> new_id((size_t)nin_old, -1);
  int32_t n_ids = 0;
  for (int64_t i = 0; i < nin_old; ++i)
    if (m->flat_of[i] >= 0) new_id[i] = n_ids++;
  // depth-first relabelling of the nodes that can still be reached; blocks follow their nodes
  std::vector<SkvNode> nodes;
  std::vector<int32_t> kids, parent, old_of_new;
  std::vector<SkvSlot> slots;
  std::vector<int32_t> tok, canon, page, n_meta, flat_of((size_t)n_ids, -1);
  std::vector<uint32_t> n_ctr, n_epoch;
  std::vector<std::pair<int32_t, int32_t>> todo;   // (old node, new parent)
  todo.push_back({0, -1});
  std::vector<std::vector<std::pair<uint64_t, int32_t>>> children;   // per new node: (hash, new child) in old table order
  while (!todo.empty()) {
    const auto [on, np] = todo.back();
    todo.pop_back();
    const SkvNode o = m->nodes[on];
    const int32_t nn = (int32_t)nodes.size();
    nodes.push_back(SkvNode{(int32_t)canon.size(), o.n_blocks, 0, 0});
    kids.push_back(0);
    parent.push_back(np);
    children.emplace_back();
    for (int32_t k = 0; k < o.n_blocks; ++k) {
      const size_t f = (size_t)o.first + k;
      flat_of[new_id[m->canon[f]]] = (int32_t)canon.size();
      canon.push_back(new_id[m->canon[f]]);
      page.push_back(m->page[f]);
      n_meta.push_back(meta[f]);
      n_epoch.push_back(epoch[f]);
      tok.insert(tok.end(), m->tok.begin() + f * 16, m->tok.begin() + (f + 1) * 16);
      n_ctr.insert(n_ctr.end(), ctr.begin() + f * SKV_CTR_STRIDE, ctr.begin() + (f + 1) * SKV_CTR_STRIDE);
    }
    if (np >= 0) {   // the hash of its first block keys the node in its parent's table
      const uint64_t h = skv_hash_block_host(&tok[(size_t)nodes[nn].first * 16]);
      children[np].push_back({h, nn});
      kids[np]++;
    }
    for (int32_t q = o.tab_cap - 1; q >= 0; --q) {
      const int32_t c = m->slots[(size_t)o.tab_off + q].child;
      if (c >= 0) todo.push_back({c, nn});
    }
  }
  std::vector<int32_t> filled(nodes.size(), 0);
  for (size_t n = 0; n < nodes.size(); ++n) {
    if (children[n].empty()) continue;
    const uint32_t cap = next_pow2((uint32_t)std::max<size_t>(4, 2 * children[n].size()));
    nodes[n].tab_off = (int32_t)slots.size();
    nodes[n].tab_cap = (int32_t)cap;
    slots.resize(slots.size() + cap, SkvSlot{0, 0, -1, 0});
    for (const auto& [h, c] : children[n]) {
      uint32_t q = (uint32_t)h & (cap - 1);
      while (slots[(size_t)nodes[n].tab_off + q].child >= 0) q = (q + 1) & (cap - 1);
      slots[(size_t)nodes[n].tab_off + q] = SkvSlot{(uint32_t)h, (uint32_t)(h >> 32), c, 0};
    }
    filled[n] = (int32_t)children[n].size();
  }
  const int64_t nb = (int64_t)canon.size();
  if (nb != m->live_blocks) return SKV_EINVAL;   // the mirror lost track of a block: refuse rather than drop it
  // write everything back; counters and epochs of the free records start from zero again
  char* base = m->base;
  const Layout& L = m->L;
  auto up = [&](size_t off, const void* src, size_t bytes) {
    return bytes ? hipMemcpyAsync(base + off, src, bytes, hipMemcpyHostToDevice, st) : hipSuccess;
  };
  SKV_HIP(up(L.tok, tok.data(), tok.size() * 4));
  SKV_HIP(up(L.page, page.data(), page.size() * 4));
  SKV_HIP(up(L.meta, n_meta.data(), n_meta.size() * 4));
  SKV_HIP(up(L.canon, canon.data(), canon.size() * 4));
  SKV_HIP(up(L.flat_of, flat_of.data(), flat_of.size() * 4));
  SKV_HIP(up(L.nodes, nodes.data(), nodes.size() * sizeof(SkvNode)));
  SKV_HIP(up(L.slots, slots.data(), slots.size() * sizeof(SkvSlot)));
  SKV_HIP(up(L.ctr, n_ctr.data(), n_ctr.size() * 4));
  SKV_HIP(up(L.epoch, n_epoch.data(), n_epoch.size() * 4));
  if (m->cap_blocks > nb) {
    const size_t n = (size_t)(m->cap_blocks - nb);
    fill_u32_kernel<<<grid_for(n * SKV_CTR_STRIDE, 256), 256, 0, st>>>(t->dev.ctr + (size_t)nb * SKV_CTR_STRIDE, n * SKV_CTR_STRIDE, 0u);
    fill_u32_kernel<<<grid_for(n, 256), 256, 0, st>>>(t->dev.epoch + nb, n, 0u);
    SKV_HIP(hipGetLastError());
  }
  SKV_HIP(hipStreamSynchronize(st));
  for (int64_t i = 0; i < nin_old; ++i) id_map[i] = new_id[i];
  m->nodes = std::move(nodes);
  m->kids = std::move(kids);
  m->filled = std::move(filled);
  m->parent = std::move(parent);
  m->slots = std::move(slots);
  m->slots_used = m->slots.size();
  m->tok = std::move(tok);
  m->canon = std::move(canon);
  m->page = std::move(page);
  m->flat_of = std::move(flat_of);
  m->vis = std::move(n_meta);   // just read back: exact
  m->node_of.assign((size_t)nb, 0);
  for (size_t n = 1; n < m->nodes.size(); ++n)
    for (int32_t k = 0; k < m->nodes[n].n_blocks; ++k) m->node_of[(size_t)m->nodes[n].first + k] = (int32_t)n;
  m->vis_stale = false;
  t->dev.n_blocks = (int32_t)nb;
  t->dev.n_nodes = (int32_t)m->nodes.size() - 1;
  t->n_in_blocks = n_ids;
  if (n_in_blocks_after) *n_in_blocks_after = n_ids;
  return SKV_OK;
}

extern "C" int skv_tree_info(const skv_tree* t, int64_t* n_nodes, int64_t* n_blocks, int64_t* n_in_blocks) {
  if (!t) return SKV_EINVAL;
  if (n_nodes) *n_nodes = t->dev.n_nodes;
  if (n_blocks) *n_blocks = t->host ? t->host->live_blocks : t->dev.n_blocks;
  if (n_in_blocks) *n_in_blocks = t->n_in_blocks;
  return SKV_OK;
}

extern "C" void skv_tree_destroy(skv_tree* t) {
  if (t) delete t->host;
  delete t;
}

extern "C" int skv_counters_read(skv_tree* t, uint32_t* d_hit, uint32_t* d_ucnt, void* stream) {
  if (!t || !d_hit || !d_ucnt) return SKV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  if (t->n_in_blocks) {
    fill_u32_kernel<<<grid_for((size_t)t->n_in_blocks, 256), 256, 0, st>>>(d_hit, (size_t)t->n_in_blocks, 0u);
    fill_u32_kernel<<<grid_for((size_t)t->n_in_blocks, 256), 256, 0, st>>>(d_ucnt, (size_t)t->n_in_blocks, 0u);
  }
  if (t->dev.n_blocks)
    counters_scatter_kernel<<<grid_for((size_t)t->dev.n_blocks, 256), 256, 0, st>>>(t->dev, d_hit, d_ucnt);
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_counters_reset(skv_tree* t, void* stream) {
  if (!t) return SKV_EINVAL;
  if (t->dev.n_blocks)
    counters_clear_window_kernel<<<grid_for((size_t)t->dev.n_blocks, 256), 256, 0, (hipStream_t)stream>>>(t->dev);
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_window_roll(skv_tree* t, const skv_rdr_policy* pol, int32_t* d_n_demoted, void* stream) {
  if (!t || !pol) return SKV_EINVAL;
  if ((pol->direction != 0 && pol->direction != 1) || pol->tau_den == 0 || pol->n_consec == 0) return SKV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  if (d_n_demoted) fill_u32_kernel<<<1, 64, 0, st>>>((uint32_t*)d_n_demoted, 1, 0u);
  if (t->dev.n_blocks)
    window_roll_kernel<<<grid_for((size_t)t->dev.n_blocks, 256), 256, 0, st>>>(t->dev, *pol, d_n_demoted);
  if (t->host) t->host->vis_stale = true;   // the kernel decides the demotions
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_promote(skv_tree* t, const int32_t* d_block_ids, int32_t n, void* stream) {
  if (!t || n < 0 || (n > 0 && !d_block_ids)) return SKV_EINVAL;
  if (n) promote_kernel<<<grid_for((size_t)n, 256), 256, 0, (hipStream_t)stream>>>(t->dev, t->n_in_blocks, d_block_ids, n);
  if (n && t->host) t->host->vis_stale = true;   // the ids are in device memory: the host has not seen them
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_block_state_read(skv_tree* t, uint8_t* d_private, uint32_t* d_hit_pre, uint32_t* d_u_pre,
                                    void* stream) {
  if (!t) return SKV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const size_t n = (size_t)t->n_in_blocks;
  if (n) {
    if (d_private) fill_u8_kernel<<<grid_for(n, 256), 256, 0, st>>>(d_private, n, (uint8_t)255);
    if (d_hit_pre) fill_u32_kernel<<<grid_for(n, 256), 256, 0, st>>>(d_hit_pre, n, 0u);
    if (d_u_pre) fill_u32_kernel<<<grid_for(n, 256), 256, 0, st>>>(d_u_pre, n, 0u);
  }
  if (t->dev.n_blocks)
    block_state_scatter_kernel<<<grid_for((size_t)t->dev.n_blocks, 256), 256, 0, st>>>(t->dev, d_private, d_hit_pre, d_u_pre);
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}
