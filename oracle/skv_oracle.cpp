// CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
//
// Plain, slow, obviously-correct statement of what the selective-reuse prefill path
// computes.  Nothing here is shared with the GPU library: no headers, no helpers, no
// tables.  Only tests, the smoke check and the benchmark's CPU-baseline leg may load it.
//
// What it follows (SafeKV paper):
//  * Unified radix-tree index with per-entry visibility metadata (Section 4.3.1,
//    "Unified Privacy-Preserving Cache Index"): a lookup walks the prefix path and checks
//    private_tag at every hop; a private entry is visible only to its creator_id; the walk
//    stops at the first entry it may not use.
//  * Access monitor (Section 4.2.2, "Safeguard"): every cache lookup records, per KV block,
//    the hit count of the current window (hit_cur) and the number of distinct tenants that
//    hit it (u_cnt); RDR = u_cnt / hit_cur (also Section 6, "Misclassification Risk and
//    Exposure Control", the RDR equation).
//  * Scaled dot-product attention with KV reuse (Section 2.1): cached K/V of the matched
//    prefix are reused, only the uncached suffix is computed; evaluated here from the
//    textbook definition in double precision.
//
// Readings taken where the paper is silent (block = 16 tokens, metadata per block, child
// key = whole first block, first insertion of a block-prefix wins, the creator's own hits
// count) are listed in the design document.
//
//  * Safeguard step (Section 4.2.2 and Section 6): at the end of a monitoring window the RDR of each
//    shareable block is tested against a threshold; a block that meets the predicate for enough
//    consecutive windows is demoted to private (visible to its creator only), then the window rolls
//    (hit_pre <- hit_cur, u_pre <- u_cnt, current counters cleared).  The paper states the trigger
//    both ways (RDR above a threshold with a narrow history, Section 4.2.2; RDR below a threshold for
//    consecutive windows, Section 6) and gives no threshold: the predicate is therefore a parameter,
//    and which direction is "right" is parity unpinned.  The mechanics for a given parameter set are
//    pinned against an independent recomputation from the counters.
//
//  * Insert after prefill (Section 4.3.1 Insert, Section 4.1 and Section 6: new blocks start private), promotion as a flag
//    flip (Section 4.2.3), per-tenant copies of the same content with a depth-first longest-visible-path search
//    (Section 4.1), access epochs and block-by-block eviction of the oldest unprotected childless tail
//    (Section 4.3.1 Evict, Section 4.3.2 progressive eviction), and the byte copy of new KV blocks into pool
//    pages.
//
// Pins (all in the CPU test-suite): brute-force prefix scans, the 0 % / 100 % sensitive special cases, the
// visibility invariants, counter conservation, closed-form / library attention cases; the safeguard step against
// an independent recomputation with exact fractions; insert, eviction and copies against models without any tree
// (a dictionary of whole block-prefixes, a flat entry list with parent links).
// Parity unpinned: WHICH safeguard policy (trigger direction, threshold) and WHICH eviction policy (tie-break,
// what counts as "in use") the paper means -- it prints no example of either; what is pinned is that the readings
// stated above are carried out exactly.

#include <array>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <map>
#include <memory>
#include <set>
#include <thread>
#include <vector>

namespace {

constexpr int kBlock = 16;
using BlockKey = std::array<int32_t, kBlock>;

struct BlockEntry {
  BlockKey tokens;
  bool is_private;      // private_tag
  int32_t creator_id;
  int32_t page_id;      // KV address of this block (address-vector entry)
  int64_t block_id;     // caller's index of the block that created this entry
  uint64_t hit_cur = 0;
  std::set<int32_t> tenants;  // distinct tenants that hit the block in the current window
  uint64_t hit_pre = 0;       // previous window
  uint64_t u_pre = 0;
  uint32_t streak = 0;        // consecutive windows in which the RDR predicate held
  uint32_t epoch = 0;         // value of the global epoch counter at the entry's last access
};

struct Node {
  std::vector<BlockEntry> blocks;               // the compressed edge: one or more blocks
  // keyed by the child's whole first block; several children may share a key (copies of the same content
  // that different tenants created while they could not see each other's), kept in creation order
  std::multimap<BlockKey, std::unique_ptr<Node>> children;
};

struct Tree {
  Node root;  // holds no blocks
  int max_node_blocks;  // 0 = unlimited (path-compressed); 1 = one block per node
  int64_t n_blocks = 0;
  uint32_t epoch = 0;   // global epoch counter (Section 4.3.2, progressive eviction)
};

BlockKey key_at(const int32_t* tok) {
  BlockKey k;
  std::memcpy(k.data(), tok, sizeof(int32_t) * kBlock);
  return k;
}

// Cut `node` after its first `keep` blocks; the remainder becomes its only child.
void split_node(Node* node, size_t keep) {
  auto tail = std::make_unique<Node>();
  tail->blocks.assign(node->blocks.begin() + keep, node->blocks.end());
  tail->children = std::move(node->children);
  node->children.clear();
  node->blocks.resize(keep);
  BlockKey k = tail->blocks[0].tokens;
  node->children.emplace(k, std::move(tail));
}

void insert_sequence(Tree* t, const int32_t* tok, int64_t n_blocks, const uint8_t* sens,
                     const int32_t* owner, const int32_t* page, int64_t first_block_id) {
  Node* node = &t->root;
  int64_t j = 0;  // next block of the sequence
  while (j < n_blocks) {
    BlockKey k = key_at(tok + j * kBlock);
    auto it = node->children.lower_bound(k);   // one copy per block-prefix in this mode: the oldest child with this key
    if (it == node->children.end() || !(it->first == k)) {
      // nothing cached below this point: append the remainder as new entries
      Node* at = node;
      while (j < n_blocks) {
        auto fresh = std::make_unique<Node>();
        int64_t take = n_blocks - j;
        if (t->max_node_blocks > 0 && take > t->max_node_blocks) take = t->max_node_blocks;
        for (int64_t i = 0; i < take; ++i, ++j) {
          BlockEntry e;
          e.tokens = key_at(tok + j * kBlock);
          e.is_private = sens[j] != 0;
          e.creator_id = owner[j];
          e.page_id = page[j];
          e.block_id = first_block_id + j;
          e.epoch = t->epoch;
          fresh->blocks.push_back(e);
          t->n_blocks++;
        }
        BlockKey fk = fresh->blocks[0].tokens;
        Node* next = fresh.get();
        at->children.emplace(fk, std::move(fresh));
        at = next;
      }
      return;
    }
    Node* child = it->second.get();
    size_t same = 0;  // blocks of the child's edge equal to the sequence
    while (same < child->blocks.size() && j + (int64_t)same < n_blocks &&
           child->blocks[same].tokens == key_at(tok + (j + same) * kBlock))
      ++same;
    // blocks already present keep their first metadata (first insertion wins)
    j += same;
    if (same < child->blocks.size()) {
      if (j == n_blocks) return;          // sequence ends inside the edge: nothing new
      split_node(child, same);            // diverges inside the edge
    }
    node = child;
  }
}

// Longest visible prefix for one request (Section 4.3.1 Search: the visibility rule is checked at every
// hop and the walk stops at the first entry the requester may not use).  Where several children start with
// the request's next block -- copies of the same content, Section 4.1: selective isolation leaves redundant
// copies -- every copy whose first block is visible is followed and the longest result kept; among equally
// long results the one found first wins, copies being tried in creation order (ascending block id).
struct PathEnd { Node* node; size_t used; };  // where a path stops: `used` blocks of `node` belong to it

struct Search {
  const int32_t* tok;
  int64_t nb;
  int32_t tenant;
  std::vector<BlockEntry*> cur, best;
  PathEnd best_end;
  bool have = false;

  void consider(Node* node, size_t used) {
    if (!have || cur.size() > best.size()) {
      best = cur;
      best_end = PathEnd{node, used};
      have = true;
    }
  }
  // `node` is fully matched (or the root); the request's next block is j
  void descend(Node* node, int64_t j) {
    bool went = false;
    if (j < nb) {
      auto range = node->children.equal_range(key_at(tok + j * kBlock));
      for (auto it = range.first; it != range.second; ++it) {
        Node* child = it->second.get();
        size_t m = 0;  // leading blocks of the child's edge that match and are visible
        while (m < child->blocks.size() && j + (int64_t)m < nb) {
          BlockEntry& e = child->blocks[m];
          if (!(e.tokens == key_at(tok + (j + m) * kBlock))) break;
          if (e.is_private && e.creator_id != tenant) break;   // visibility rule, every hop
          ++m;
        }
        if (m == 0) continue;
        went = true;
        for (size_t i = 0; i < m; ++i) cur.push_back(&child->blocks[i]);
        if (m == child->blocks.size()) descend(child, j + (int64_t)m);
        else consider(child, m);
        cur.resize(cur.size() - m);
        if ((int64_t)best.size() == nb) return;   // cannot get longer
      }
    }
    if (!went) consider(node, node->blocks.size());
  }
};

int64_t match_one(Tree* t, const int32_t* tok, int64_t n_tokens, int32_t tenant,
                  std::vector<BlockEntry*>* out, PathEnd* end = nullptr) {
  Search s{tok, n_tokens / kBlock, tenant, {}, {}, PathEnd{&t->root, 0}};  // a trailing partial block never matches
  s.descend(&t->root, 0);
  *out = s.best;
  if (end) *end = s.best_end;
  return (int64_t)s.best.size();
}

void for_each_block(Node* n, const std::function<void(BlockEntry&)>& f) {
  for (auto& b : n->blocks) f(b);
  for (auto& kv : n->children) for_each_block(kv.second.get(), f);
}
int64_t count_nodes(Node* n) {
  int64_t c = 1;
  for (auto& kv : n->children) c += count_nodes(kv.second.get());
  return c;
}

inline double load_elem(const void* base, int dtype, int64_t idx) {
  if (dtype == 0) return (double)((const float*)base)[idx];
  uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;  // bf16 -> fp32, exact
  float f;
  std::memcpy(&f, &bits, 4);
  return (double)f;
}

struct AttnArgs {
  int dtype, Hq, Hkv, d;
  double scale;
  const int32_t* q_off;
  const void *q, *knew, *vnew, *kpool, *vpool;
  const int32_t* matched_len;
  const int32_t* page_table;
  int max_blocks;
};

// One output row: request r, query head h, suffix position i.
void attention_row(const AttnArgs& a, int r, int h, int i, double* out) {
  const int d = a.d, G = a.Hq / a.Hkv, hk = h / G;
  const int64_t L = a.matched_len[r];
  const int64_t n_keys = L + i + 1;  // whole reused prefix, then own positions 0..i
  const int64_t qrow = ((int64_t)a.q_off[r] + i) * a.Hq + h;
  std::vector<double> logit(n_keys);
  double m = -INFINITY;
  for (int64_t j = 0; j < n_keys; ++j) {
    const void* kb;
    int64_t kidx;
    if (j < L) {
      int64_t page = a.page_table[(int64_t)r * a.max_blocks + j / kBlock];
      kb = a.kpool;
      kidx = ((page * kBlock + j % kBlock) * a.Hkv + hk) * d;
    } else {
      kb = a.knew;
      kidx = (((int64_t)a.q_off[r] + (j - L)) * a.Hkv + hk) * d;
    }
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += load_elem(a.q, a.dtype, qrow * d + c) * load_elem(kb, a.dtype, kidx + c);
    logit[j] = a.scale * s;
    if (logit[j] > m) m = logit[j];
  }
  double denom = 0.0;
  std::vector<double> acc(d, 0.0);
  for (int64_t j = 0; j < n_keys; ++j) {
    const double p = std::exp(logit[j] - m);
    denom += p;
    const void* vb;
    int64_t vidx;
    if (j < L) {
      int64_t page = a.page_table[(int64_t)r * a.max_blocks + j / kBlock];
      vb = a.vpool;
      vidx = ((page * kBlock + j % kBlock) * a.Hkv + hk) * d;
    } else {
      vb = a.vnew;
      vidx = (((int64_t)a.q_off[r] + (j - L)) * a.Hkv + hk) * d;
    }
    for (int c = 0; c < d; ++c) acc[c] += p * load_elem(vb, a.dtype, vidx + c);
  }
  for (int c = 0; c < d; ++c) out[c] = acc[c] / denom;
}

}  // namespace

extern "C" {

void* okv_tree_new(int max_node_blocks) {
  Tree* t = new Tree();
  t->max_node_blocks = max_node_blocks;
  return t;
}
void okv_tree_free(void* t) { delete (Tree*)t; }

// Insert cached sequences.  seq_off are token offsets (multiples of 16); the per-block arrays
// are indexed by the block's position in the concatenated input (its "block id").
int okv_tree_insert(void* tp, int64_t n_seq, const int64_t* seq_off, const int32_t* tokens,
                    const uint8_t* sens, const int32_t* owner, const int32_t* page) {
  Tree* t = (Tree*)tp;
  for (int64_t s = 0; s < n_seq; ++s) {
    int64_t lo = seq_off[s], hi = seq_off[s + 1];
    if (lo % kBlock || hi % kBlock || hi < lo) return -1;
    int64_t b0 = lo / kBlock;
    insert_sequence(t, tokens + lo, (hi - lo) / kBlock, sens + b0, owner + b0, page + b0, b0);
  }
  return 0;
}

// Blocks of a token sequence that already lie on a root path (tokens only; visibility plays no part).
int64_t existing_prefix_blocks(Tree* t, const int32_t* tok, int64_t n_blocks) {
  Node* node = &t->root;
  int64_t j = 0;
  while (j < n_blocks) {
    const BlockKey k = key_at(tok + j * kBlock);
    auto it = node->children.lower_bound(k);
    if (it == node->children.end() || !(it->first == k)) return j;
    Node* child = it->second.get();
    for (size_t i = 0; i < child->blocks.size(); ++i) {
      if (j == n_blocks || !(child->blocks[i].tokens == key_at(tok + j * kBlock))) return j;
      ++j;
    }
    node = child;
  }
  return j;
}

// Insert after a prefill (Section 4.3.1 Insert; Section 4.1 and Section 6: every new block starts private): the full
// blocks of request r that the tree does not hold yet are appended along its path with private_tag = 1 and
// creator_id = the request's tenant.  One copy per block-prefix: blocks whose tokens are already on the path
// keep their entry, whoever created it.  new_pages[r][j] is the page of the request's block
// matched_len[r]/16 + j (the pages its suffix was written to); insertion stops at the first block without
// a page (< 0 or beyond max_new_blocks).  New entries get the ids next_block_id, next_block_id+1, ... in
// request order.  Per request: first_inserted = index of its first new block, n_inserted = how many.
// Returns the next free block id.
//
// private_copies != 0 (Section 4.1: selective isolation leaves redundant copies): a requester that is stopped
// by an entry it may not see adds its own copy instead.  The request's longest visible path is looked up in
// the tree as it stands (requests are handled in order), and all of its full blocks beyond that path are
// appended below the path's end, private to the tenant -- next to whatever other tenants cached there.
int64_t okv_insert_requests(void* tp, int32_t n_req, const int32_t* req_off, const int32_t* req_tokens,
                            const int32_t* req_tenant, const int32_t* matched_len, const int32_t* new_pages,
                            int32_t max_new_blocks, int64_t next_block_id, int32_t* first_inserted,
                            int32_t* n_inserted, int32_t private_copies) {
  Tree* t = (Tree*)tp;
  for (int32_t r = 0; r < n_req; ++r) {
    const int32_t* tok = req_tokens + req_off[r];
    int64_t nb = (req_off[r + 1] - req_off[r]) / kBlock;
    const int64_t k_vis = matched_len[r] / kBlock;
    int64_t have = 0;  // leading suffix blocks that come with a page
    while (have < max_new_blocks && new_pages[(int64_t)r * max_new_blocks + have] >= 0) ++have;
    if (nb > k_vis + have) nb = k_vis + have;
    if (private_copies) {
      std::vector<BlockEntry*> path;
      PathEnd end{&t->root, 0};
      const int64_t k = match_one(t, tok, nb * kBlock, req_tenant[r], &path, &end);
      first_inserted[r] = (int32_t)k;
      n_inserted[r] = 0;
      if (k >= nb || k < k_vis) continue;
      if (end.used < end.node->blocks.size()) split_node(end.node, end.used);  // the path stops inside a compressed edge
      auto fresh = std::make_unique<Node>();
      for (int64_t j = k; j < nb; ++j) {
        BlockEntry e;
        e.tokens = key_at(tok + j * kBlock);
        e.is_private = true;
        e.creator_id = req_tenant[r];
        e.page_id = new_pages[(int64_t)r * max_new_blocks + (j - k_vis)];
        e.block_id = next_block_id++;
        e.epoch = t->epoch;
        fresh->blocks.push_back(e);
        t->n_blocks++;
      }
      const BlockKey fk = fresh->blocks[0].tokens;
      end.node->children.emplace(fk, std::move(fresh));
      n_inserted[r] = (int32_t)(nb - k);
      continue;
    }
    const int64_t k_exist = existing_prefix_blocks(t, tok, nb);
    first_inserted[r] = (int32_t)k_exist;
    n_inserted[r] = 0;
    if (k_exist >= nb || k_exist < k_vis) continue;  // nothing new, or a matched length the tree cannot have given
    std::vector<uint8_t> sens(nb, 1);
    std::vector<int32_t> owner(nb, req_tenant[r]), page(nb, -1);
    for (int64_t j = k_vis; j < nb; ++j) page[j] = new_pages[(int64_t)r * max_new_blocks + (j - k_vis)];
    insert_sequence(t, tok, nb, sens.data(), owner.data(), page.data(), next_block_id - k_exist);
    n_inserted[r] = (int32_t)(nb - k_exist);
    next_block_id += nb - k_exist;
  }
  return next_block_id;
}

// Eviction (Section 4.3.1 Evict: epoch-based LRU, entries in use are protected; Section 4.3.2: space is
// reclaimed from leaf to root, a compressed chain gives up the entries of its address vector one at a time
// from its far end and disappears only when the vector is empty).  Only the last block of a childless node
// can go without cutting off other entries; among those candidates that are not protected the one with the
// oldest access epoch goes first (ties: the smaller block id), and the choice is repeated until n_want
// blocks are gone or no candidate is left.  Writes the evicted block ids and their pages in eviction order.
void okv_set_epoch(void* tp, uint32_t e) { ((Tree*)tp)->epoch = e; }

void okv_block_epochs(void* tp, int64_t n_in_blocks, uint32_t* epoch) {
  for (int64_t i = 0; i < n_in_blocks; ++i) epoch[i] = 0;
  for_each_block(&((Tree*)tp)->root, [&](BlockEntry& e) { epoch[e.block_id] = e.epoch; });
}

struct Victim { Node* node = nullptr; Node* parent = nullptr; };
void find_victim(Node* n, const std::set<int64_t>& prot, Victim* best) {
  for (auto& kv : n->children) {
    Node* c = kv.second.get();
    if (c->children.empty() && !c->blocks.empty()) {
      const BlockEntry& tail = c->blocks.back();
      if (!prot.count(tail.block_id)) {
        bool better = !best->node;
        if (!better) {
          const BlockEntry& b = best->node->blocks.back();
          better = tail.epoch < b.epoch || (tail.epoch == b.epoch && tail.block_id < b.block_id);
        }
        if (better) { best->node = c; best->parent = n; }
      }
    }
    find_victim(c, prot, best);
  }
}

int64_t okv_evict(void* tp, int64_t n_want, int64_t n_protect, const int64_t* protect, int64_t* out_ids,
                  int32_t* out_pages) {
  Tree* t = (Tree*)tp;
  std::set<int64_t> prot(protect, protect + n_protect);
  int64_t done = 0;
  while (done < n_want) {
    Victim v;
    find_victim(&t->root, prot, &v);
    if (!v.node) break;
    const BlockEntry gone = v.node->blocks.back();
    out_ids[done] = gone.block_id;
    out_pages[done] = gone.page_id;
    ++done;
    v.node->blocks.pop_back();
    t->n_blocks--;
    if (v.node->blocks.empty()) {  // it was the node's first block: the node leaves its parent
      auto range = v.parent->children.equal_range(gone.tokens);
      for (auto it = range.first; it != range.second; ++it)
        if (it->second.get() == v.node) { v.parent->children.erase(it); break; }
    }
  }
  return done;
}

int64_t okv_tree_n_blocks(void* tp) { return ((Tree*)tp)->n_blocks; }
int64_t okv_tree_n_nodes(void* tp) { return count_nodes(&((Tree*)tp)->root) - 1; }

// Match a batch sequentially.  page_table is [n_req, max_blocks] (-1 beyond the match),
// block_ids likewise (may be null).  update != 0 records the hits in the access monitor.
int okv_match(void* tp, int32_t n_req, const int32_t* req_off, const int32_t* req_tokens,
              const int32_t* req_tenant, int32_t max_blocks, int32_t* matched_len,
              int32_t* page_table, int64_t* block_ids, int update) {
  Tree* t = (Tree*)tp;
  for (int32_t r = 0; r < n_req; ++r) {
    std::vector<BlockEntry*> hits;
    int64_t n_tok = req_off[r + 1] - req_off[r];
    if (n_tok / kBlock > max_blocks) n_tok = (int64_t)max_blocks * kBlock;
    int64_t k = match_one(t, req_tokens + req_off[r], n_tok, req_tenant[r], &hits);
    matched_len[r] = (int32_t)(k * kBlock);
    for (int32_t j = 0; j < max_blocks; ++j) {
      page_table[(int64_t)r * max_blocks + j] = j < k ? hits[j]->page_id : -1;
      if (block_ids) block_ids[(int64_t)r * max_blocks + j] = j < k ? hits[j]->block_id : -1;
    }
    if (update)
      for (BlockEntry* e : hits) {
        e->hit_cur += 1;
        e->tenants.insert(req_tenant[r]);
        e->epoch = t->epoch;
      }
  }
  return 0;
}

// Counters of the current window, indexed by block id; entries of blocks that created no
// tree entry (repeats of an already cached block-prefix) stay 0.
void okv_counters(void* tp, int64_t n_in_blocks, uint32_t* hit, uint32_t* u_cnt) {
  std::memset(hit, 0, sizeof(uint32_t) * n_in_blocks);
  std::memset(u_cnt, 0, sizeof(uint32_t) * n_in_blocks);
  for_each_block(&((Tree*)tp)->root, [&](BlockEntry& e) {
    hit[e.block_id] = (uint32_t)e.hit_cur;
    u_cnt[e.block_id] = (uint32_t)e.tenants.size();
  });
}

// The single tenant recorded for a block, or -1 if none / -2 if several (for the test of the
// "sensitive block is only ever hit by its owner" property).
void okv_sole_tenant(void* tp, int64_t n_in_blocks, int32_t* who) {
  for (int64_t i = 0; i < n_in_blocks; ++i) who[i] = -1;
  for_each_block(&((Tree*)tp)->root, [&](BlockEntry& e) {
    who[e.block_id] = e.tenants.empty() ? -1 : (e.tenants.size() == 1 ? *e.tenants.begin() : -2);
  });
}

// Safeguard step at a window boundary.  direction 0: predicate = RDR < tau (Section 6); direction 1:
// predicate = RDR > tau and u_pre <= u_pre_max (Section 4.2.2).  RDR = u_cnt / hit_cur is compared as
// the exact rational: u_cnt * tau_den (<|>) tau_num * hit_cur.  Blocks with hit_cur < min_hits do not
// meet the predicate.  A shareable block whose predicate has held for n_consec consecutive windows
// (this one included) is demoted.  Returns the number of blocks demoted.
int64_t okv_window_roll(void* tp, int direction, uint32_t tau_num, uint32_t tau_den, uint32_t min_hits,
                        uint32_t n_consec, uint32_t u_pre_max) {
  int64_t demoted = 0;
  for_each_block(&((Tree*)tp)->root, [&](BlockEntry& e) {
    const uint64_t u = e.tenants.size(), h = e.hit_cur;
    bool pred = false;
    if (h > 0 && h >= min_hits) {
      if (direction == 0) pred = u * tau_den < (uint64_t)tau_num * h;
      else pred = u * tau_den > (uint64_t)tau_num * h && e.u_pre <= u_pre_max;
    }
    e.streak = pred ? e.streak + 1 : 0;
    if (!e.is_private && e.streak >= n_consec) {
      e.is_private = true;   // creator_id is already recorded: from now on only the creator may reuse it
      e.streak = 0;
      ++demoted;
    }
    e.hit_pre = h;
    e.u_pre = u;
    e.hit_cur = 0;
    e.tenants.clear();
  });
  return demoted;
}

// Promotion (Section 4.2.3: once a block is verified shareable its visibility bit is flipped): the
// entries created by the listed input block ids become shareable.  Ids that created no entry are ignored.
void okv_promote(void* tp, int64_t n, const int64_t* block_ids) {
  std::set<int64_t> ids(block_ids, block_ids + n);
  for_each_block(&((Tree*)tp)->root, [&](BlockEntry& e) {
    if (ids.count(e.block_id)) e.is_private = false;
  });
}

// Insert side of the KV pool (Section 4.3.1 Insert: newly generated KV blocks are appended): the full
// 16-token blocks of request r's uncached suffix are written to the pages new_pages[r][j]; entries < 0
// or beyond the suffix's full blocks are skipped.  row_bytes = bytes of one token row (all kv heads).
void okv_scatter(int64_t row_bytes, int32_t n_req, const int32_t* q_off, const int32_t* new_pages,
                 int32_t max_new_blocks, const void* knew, const void* vnew, void* kpool, void* vpool) {
  const int64_t page_bytes = row_bytes * kBlock;
  for (int32_t r = 0; r < n_req; ++r) {
    const int32_t full = (q_off[r + 1] - q_off[r]) / kBlock;
    for (int32_t j = 0; j < full && j < max_new_blocks; ++j) {
      const int64_t p = new_pages[(int64_t)r * max_new_blocks + j];
      if (p < 0) continue;
      const int64_t src = ((int64_t)q_off[r] + (int64_t)j * kBlock) * row_bytes;
      std::memcpy((char*)kpool + p * page_bytes, (const char*)knew + src, page_bytes);
      std::memcpy((char*)vpool + p * page_bytes, (const char*)vnew + src, page_bytes);
    }
  }
}

// Per input block id: private_tag (0 / 1) of the entry it created, 255 for blocks that created none;
// previous-window counters likewise (0 for blocks that created none).
void okv_block_state(void* tp, int64_t n_in_blocks, uint8_t* is_private, uint32_t* hit_pre, uint32_t* u_pre) {
  for (int64_t i = 0; i < n_in_blocks; ++i) { is_private[i] = 255; hit_pre[i] = 0; u_pre[i] = 0; }
  for_each_block(&((Tree*)tp)->root, [&](BlockEntry& e) {
    is_private[e.block_id] = e.is_private ? 1 : 0;
    hit_pre[e.block_id] = (uint32_t)e.hit_pre;
    u_pre[e.block_id] = (uint32_t)e.u_pre;
  });
}

void okv_counters_reset(void* tp) {
  for_each_block(&((Tree*)tp)->root, [&](BlockEntry& e) {
    e.hit_cur = 0;
    e.tenants.clear();
  });
}

// Gather: copy the matched pages of K and V into per-request contiguous staging, requests
// back to back.  elem_bytes * page_elems bytes per page.
void okv_gather(int64_t page_bytes, int32_t n_req, const int32_t* matched_len,
                const int32_t* page_table, int32_t max_blocks, const void* kpool,
                const void* vpool, void* kctx, void* vctx) {
  int64_t o = 0;
  for (int32_t r = 0; r < n_req; ++r)
    for (int32_t j = 0; j < matched_len[r] / kBlock; ++j, ++o) {
      int64_t p = page_table[(int64_t)r * max_blocks + j];
      std::memcpy((char*)kctx + o * page_bytes, (const char*)kpool + p * page_bytes, page_bytes);
      std::memcpy((char*)vctx + o * page_bytes, (const char*)vpool + p * page_bytes, page_bytes);
    }
}

// Attention.  dtype 0 = fp32, 1 = bf16 (raw 16-bit).  If n_rows < 0 every (token, head) row is
// computed into out[sum S][Hq][d]; otherwise the listed rows into out[n_rows][d].
int okv_attention(int dtype, int Hq, int Hkv, int d, double scale, int32_t n_req,
                  const int32_t* q_off, const void* q, const void* knew, const void* vnew,
                  const void* kpool, const void* vpool, const int32_t* matched_len,
                  const int32_t* page_table, int32_t max_blocks, int64_t n_rows,
                  const int32_t* row_req, const int32_t* row_head, const int32_t* row_pos,
                  double* out, int n_threads) {
  if (Hq % Hkv) return -1;
  AttnArgs a{dtype, Hq, Hkv, d, scale, q_off, q, knew, vnew, kpool, vpool, matched_len,
             page_table, max_blocks};
  std::vector<std::array<int32_t, 3>> rows;
  if (n_rows < 0) {
    for (int32_t r = 0; r < n_req; ++r)
      for (int32_t i = 0; i < q_off[r + 1] - q_off[r]; ++i)
        for (int32_t h = 0; h < Hq; ++h) rows.push_back({r, h, i});
  } else {
    for (int64_t x = 0; x < n_rows; ++x) rows.push_back({row_req[x], row_head[x], row_pos[x]});
  }
  auto work = [&](int tid, int nt) {
    for (size_t x = tid; x < rows.size(); x += nt) {
      int r = rows[x][0], h = rows[x][1], i = rows[x][2];
      double* o = n_rows < 0 ? out + (((int64_t)q_off[r] + i) * Hq + h) * d : out + (int64_t)x * d;
      attention_row(a, r, h, i, o);
    }
  };
  if (n_threads <= 1) {
    work(0, 1);
  } else {
    std::vector<std::thread> th;
    for (int t = 0; t < n_threads; ++t) th.emplace_back(work, t, n_threads);
    for (auto& x : th) x.join();
  }
  return 0;
}

}  // extern "C"
