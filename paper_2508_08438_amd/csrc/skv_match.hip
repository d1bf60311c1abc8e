// Longest visible prefix match + access-monitor update, one workgroup of four wavefronts per request.
//
// SafeKV Section 4.3.1 (Search): the lookup walks the prefix path and checks private_tag at
// every hop; a private entry may only be used by its creator_id, otherwise the walk stops.
// Section 4.3.2: at a compressed node the walk reads the KV addresses from the node's address
// vector instead of chasing one pointer per block.  Section 4.2.2: every lookup records per
// KV block the hit count and the distinct tenants of the current window.
//
// Mapping to the wavefront: lane i compares request token i with tree token i of a window of
// the node's contiguous token span; a ballot of the mismatches gives the first block that
// differs, a second ballot over the blocks' metadata gives the first block the tenant may
// not see; the smaller of the two ends the walk.  The lanes of the matched blocks then copy
// the page ids and issue the counter atomics.  The four wavefronts of a workgroup take
// disjoint parts of a long node's span and combine their stop positions through LDS.
#include "skv_internal.h"

namespace {

constexpr int kWave = 64;
constexpr int kWavesPerWg = 4;
constexpr int kSub = 4;                    // 256-token sub-windows per step: one 16-byte vector (4 tokens) per lane each
constexpr int kFirstBlocks = 16;           // blocks the first round of a walk compares (one wavefront per request)
constexpr int kStepBlocks = kSub * 16;     // 64 blocks (1024 tokens) per step: one block per lane for metadata and page ids
constexpr int kAhead = 4;                  // steps of a node whose loads are in flight together
constexpr int kCoopMaxRequests = 512;      // batches up to this size give every request a whole workgroup
typedef int32_t tok4 __attribute__((ext_vector_type(4), aligned(4)));   // request offsets are token-, not 16-byte aligned

__device__ inline uint64_t ballot64(bool p) { return __ballot(p); }

__device__ inline int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ inline bool differ(tok4 p, tok4 q) { return ((p.x ^ q.x) | (p.y ^ q.y) | (p.z ^ q.z) | (p.w ^ q.w)) != 0; }

// 64-bit hash of the 16-token block starting at x (all lanes return the same value)
__device__ inline uint64_t hash_block(const int32_t* x, int lane) {
  uint64_t v = 0;
  if (lane < 16) v = skv_mix_tok((uint32_t)x[lane], (uint32_t)lane);
  for (int o = 8; o >= 1; o >>= 1) {
    uint32_t lo = __shfl_xor((uint32_t)v, o, 16);
    uint32_t hi = __shfl_xor((uint32_t)(v >> 32), o, 16);
    v += ((uint64_t)hi << 32) | lo;
  }
  v = skv_hash_fin(v);
  uint32_t lo = (uint32_t)uniform((int)(uint32_t)v);
  uint32_t hi = (uint32_t)uniform((int)(uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}

// true iff the 16 tokens at a and b are equal (wave-uniform result)
__device__ inline bool block_equal(const int32_t* a, const int32_t* b, int lane) {
  bool ne = lane < 16 && a[lane] != b[lane];
  return ballot64(ne) == 0;
}

// child of `nd` whose first block equals the request block at x, or -1
__device__ inline int find_child(const SkvTreeDev& t, const SkvNode nd, const int32_t* x, int lane) {
  if (nd.tab_cap == 0) return -1;
  const uint64_t h = hash_block(x, lane);
  const uint32_t mask = (uint32_t)nd.tab_cap - 1u;
  for (int base = 0; base < nd.tab_cap; base += kWave) {
    const bool valid = base + lane < nd.tab_cap;
    SkvSlot e{0, 0, -1, 0};
    if (valid) e = t.slots[nd.tab_off + (((uint32_t)h + (uint32_t)(base + lane)) & mask)];
    const uint64_t empty = ballot64(valid && e.child == -1);  // a removed entry (-2) does not end the probe
    uint64_t cand = ballot64(valid && e.child >= 0 && e.hash_lo == (uint32_t)h && e.hash_hi == (uint32_t)(h >> 32));
    if (empty) cand &= (empty & (~empty + 1)) - 1;  // only slots probed before the first empty one
    while (cand) {
      const int l = __builtin_ctzll(cand);
      const int child = __shfl(e.child, l);
      const int cfirst = uniform(t.nodes[child].first);
      if (block_equal(x, t.tok + (size_t)cfirst * 16, lane)) return child;
      cand &= cand - 1;  // same hash, different tokens: keep probing
    }
    if (empty) return -1;
  }
  return -1;
}

// kCoop = kWavesPerWg: one workgroup of four wavefronts per request (few requests: their long nodes set the time).
// kCoop = 1: one wavefront per request, four requests per workgroup, no exchange (many requests: throughput).
// In the cooperative form all four walk the same path (each finds the same child at a node:
// no exchange needed); a node's span is compared in rounds of kWavesPerWg groups of kAhead steps, one group per
// wavefront, whose first mismatch or invisible block is combined through LDS into the round's stop position.  Each
// wavefront then records (page ids, counters, epochs) the blocks of its own group that lie before that position.
// Every branch around a barrier depends only on values that are equal in all four wavefronts.
template <int kCoop>
__global__ __launch_bounds__(kWave* kWavesPerWg) void skv_match_kernel(
    SkvTreeDev t, int n_req, const int32_t* __restrict__ req_off, const int32_t* __restrict__ req_tok,
    const int32_t* __restrict__ req_tenant, int max_blocks, int32_t* __restrict__ matched_len,
    int32_t* __restrict__ page_table, int32_t* __restrict__ path_end) {
  __shared__ int stop_at[2][kWavesPerWg];   // per round parity and wavefront: blocks of the node matched before its stop
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = kCoop > 1 ? uniform(threadIdx.x >> 6) : 0;   // wavefront within the request's team
  const int r = kCoop > 1 ? blockIdx.x : blockIdx.x * kWavesPerWg + (threadIdx.x >> 6);
  if (kCoop == 1 && r >= n_req) return;  // whole wave leaves; this form has no barriers
  const int lo = uniform(req_off[r]), hi = uniform(req_off[r + 1]);
  const int tenant = uniform(req_tenant[r]);
  int nb = hi > lo ? (hi - lo) / SKV_BLOCK_TOKENS : 0;
  if (nb > max_blocks) nb = max_blocks;
  if (tenant < 0 || tenant >= t.n_tenants) nb = 0;
  const int32_t* x = req_tok + lo;
  int32_t* row = page_table + (size_t)r * max_blocks;
  const uint32_t tbit = 1u << (tenant & 31);
  const int tword = 1 + (tenant >> 5);
  constexpr int kGroup = kAhead * kStepBlocks;        // blocks one wavefront compares per round
  constexpr int kRound = kCoop * kGroup;

  int j = 0;      // blocks matched so far
  int node = 0;   // current node (root)
  int last = -1;  // record of the last matched block: where the path ends
  int parity = 0;
  bool stop = false;
  while (j < nb && !stop) {
    SkvNode cur = t.nodes[node];
    cur.tab_off = uniform(cur.tab_off);
    cur.tab_cap = uniform(cur.tab_cap);
    const int child = find_child(t, cur, x + (size_t)j * 16, lane);
    if (child < 0) break;
    SkvNode nd = t.nodes[child];
    const int first = uniform(nd.first);
    const int nblk = uniform(nd.n_blocks);
    const int span = min(nblk, nb - j);  // blocks of this node the request can still cover
    const int jn = j;                    // request block that faces the node's first block
    // With one wavefront per request (large batches) the very first round of a walk looks at kFirstBlocks blocks only:
    // where sensitive blocks are frequent most walks end within a few blocks, and a full round would have fetched a
    // few hundred blocks of the node for them.  A walk that gets past them pays one more round trip.
    int width = (kCoop == 1 && j == 0) ? kFirstBlocks : kRound;
    for (int r0 = 0; r0 < span && !stop; r0 += width, width = kRound) {
      // A node's span is contiguous, so the addresses of all steps are known at once: the loads of this wavefront's
      // kAhead steps (tokens of both sides, metadata, page ids) are issued together, then compared.
      const int g0 = r0 + wave * kGroup;            // first block (within the node) of this wavefront's group
      const int g1 = min(span, g0 + (kCoop == 1 ? width : kGroup));
      tok4 a[kAhead][kSub], b[kAhead][kSub];
      int m[kAhead], pg[kAhead];   // per-block metadata word and page id of the lane's block
#pragma unroll
      for (int s = 0; s < kAhead; ++s) {
        const int c = g0 + s * kStepBlocks;
        if (c < g1) {
          const int cb = min(kStepBlocks, g1 - c);
          const int ntok = cb * 16;
          const tok4* tt = (const tok4*)(t.tok + (size_t)(first + c) * 16);
          const tok4* xx = (const tok4*)(x + (size_t)(jn + c) * 16);
          const tok4 z = {0, 0, 0, 0};
#pragma unroll
          for (int u = 0; u < kSub; ++u) {
            const int i = u * kWave + lane;      // vector index: tokens 4 i .. 4 i + 3, block i / 4
            a[s][u] = 4 * i < ntok ? xx[i] : z;
            b[s][u] = 4 * i < ntok ? tt[i] : z;
          }
          m[s] = lane < cb ? t.meta[first + c + lane] : 0;
          pg[s] = lane < cb ? t.page[first + c + lane] : 0;
        }
      }
      int good = g1 > g0 ? g1 - g0 : 0;   // leading blocks of the group that match and are visible
      bool open = true;
#pragma unroll
      for (int s = 0; s < kAhead; ++s) {
        const int c = g0 + s * kStepBlocks;
        if (c < g1 && open) {
          const int cb = min(kStepBlocks, g1 - c);
          int n_eq = cb;  // leading blocks whose tokens all agree
#pragma unroll
          for (int u = kSub - 1; u >= 0; --u) {
            const uint64_t ne = ballot64(differ(a[s][u], b[s][u]));
            if (ne) n_eq = u * 16 + (__builtin_ctzll(ne) >> 2);
          }
          // visibility rule: private (bit 31) entries only for their creator
          const uint64_t hidden = ballot64(m[s] < 0 && (m[s] & 0x7fffffff) != tenant);
          const int n_vis = hidden ? __builtin_ctzll(hidden) : cb;
          const int take = min(n_eq, n_vis);
          if (take < cb) {
            good = s * kStepBlocks + take;
            open = false;
          }
        }
      }
      // the round's stop: the first group that ends early ends the walk there
      int upto = r0;         // blocks of the node matched once this round is done
      bool ended = false;
      if (kCoop > 1) {
        if (lane == 0) stop_at[parity][wave] = good;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kCoop; ++w) {
          const int w0 = r0 + w * kGroup, w1 = min(span, w0 + kGroup);
          if (!ended && w0 < span) {
            const int gw = stop_at[parity][w];
            upto = w0 + gw;
            if (gw < w1 - w0) ended = true;
          }
        }
        parity ^= 1;         // the other row takes the next round: no second barrier is needed
      } else {
        upto = g0 + good;
        ended = good < g1 - g0;
      }
      // record this wavefront's blocks that lie before the stop
      const int mine = min(upto, g1) - g0;
#pragma unroll
      for (int s = 0; s < kAhead; ++s) {
        const int c = g0 + s * kStepBlocks;
        if (c + lane < g0 + mine) {
          const int blk = first + c + lane;
          row[jn + c + lane] = pg[s];
          uint32_t* ctr = t.ctr + (size_t)blk * SKV_CTR_STRIDE;
          atomicAdd(ctr, 1u);
          atomicOr(ctr + tword, tbit);
          t.epoch[blk] = t.cur_epoch;  // every lookup of one batch writes the same value
        }
      }
      j = jn + upto;
      if (upto > 0) last = first + upto - 1;
      if (ended) stop = true;
    }
    node = child;
  }
  if (wave == 0 && lane == 0) {
    matched_len[r] = j * SKV_BLOCK_TOKENS;
    if (path_end) path_end[r] = last;
  }
  for (int i = j + wave * kWave + lane; i < max_blocks; i += kWave * kCoop) row[i] = -1;
}

// ---- lookup on a tree with per-tenant copies ---------------------------------------------------------
// (Section 4.1: selective isolation leaves redundant copies of the same content.)  A position may then hold
// several children that start with the request's next block, and the longest visible path can run through
// any copy whose first block the tenant may see.  One wavefront still owns a request; it walks the tree
// once per combination of choices, in lexicographic order of the choices (copies ordered by the input block
// id of their first block), and keeps the first of the longest walks -- the order in which a depth-first
// search that tries older copies first meets them.  A walk is described by up to kMaxChoice 6-bit ranks
// packed into one 64-bit word; past that many branch points the oldest visible copy is taken without alternatives,
// of more than kMaxCopies visible copies at one position the kMaxCopies oldest are considered, and at most kMaxWalks
// walks are made.  A request that runs into one of these limits may get a shorter path than the longest one; the
// limit's bit is then set in the tree's limits word (skv_match_limits_read), so the caller knows.
constexpr int kMaxChoice = 10;
constexpr int kMaxCopies = 64;
constexpr int kMaxWalks = 4096;

// The `want`-th oldest child of `nd` whose first block equals the request block at x and is visible to the
// tenant; *n_out = how many such children there are.  -1 if none.
__device__ inline int find_child_ranked(const SkvTreeDev& t, const SkvNode nd, const int32_t* x, int tenant, int lane,
                                        int want, int* n_out, uint32_t* limits) {
  *n_out = 0;
  if (nd.tab_cap == 0) return -1;
  const uint64_t h = hash_block(x, lane);
  const uint32_t mask = (uint32_t)nd.tab_cap - 1u;
  int n = 0;                       // candidates so far (uniform); candidate i lives in lane i
  int my_canon = 0x7fffffff, my_child = -1;
  for (int base = 0; base < nd.tab_cap; base += kWave) {
    const bool valid = base + lane < nd.tab_cap;
    SkvSlot e{0, 0, -1, 0};
    if (valid) e = t.slots[nd.tab_off + (((uint32_t)h + (uint32_t)(base + lane)) & mask)];
    const uint64_t empty = ballot64(valid && e.child == -1);
    uint64_t cand = ballot64(valid && e.child >= 0 && e.hash_lo == (uint32_t)h && e.hash_hi == (uint32_t)(h >> 32));
    if (empty) cand &= (empty & (~empty + 1)) - 1;
    while (cand) {
      const int l = __builtin_ctzll(cand);
      const int child = __shfl(e.child, l);
      const int cfirst = uniform(t.nodes[child].first);
      if (block_equal(x, t.tok + (size_t)cfirst * 16, lane)) {
        const int m = uniform(t.meta[cfirst]);
        const bool visible = !(m < 0 && (m & 0x7fffffff) != tenant);
        if (visible) {
          const int id = uniform(t.canon[cfirst]);
          if (n < kMaxCopies) {
            if (lane == n) { my_canon = id; my_child = child; }
            ++n;
          } else {   // more copies than lanes: keep the kMaxCopies oldest, and say so
            *limits |= SKV_LIMIT_COPIES;
            int worst = my_canon;
            for (int o = 32; o >= 1; o >>= 1) worst = max(worst, __shfl_xor(worst, o));
            if (id < worst) {
              const uint64_t holder = ballot64(my_canon == worst);
              if (lane == __builtin_ctzll(holder)) { my_canon = id; my_child = child; }
            }
          }
        }
      }
      cand &= cand - 1;
    }
    if (empty) break;
  }
  *n_out = n;
  if (n == 0) return -1;
  int rank = 0;                    // how many candidates are older than this lane's
  for (int i = 0; i < n; ++i) rank += __shfl(my_canon, i) < my_canon ? 1 : 0;
  if (want >= n) want = 0;
  const uint64_t sel = ballot64(lane < n && rank == want);
  return __shfl(my_child, __builtin_ctzll(sel));
}

__global__ __launch_bounds__(kWave* kWavesPerWg) void skv_match_copies_kernel(
    SkvTreeDev t, int n_req, const int32_t* __restrict__ req_off, const int32_t* __restrict__ req_tok,
    const int32_t* __restrict__ req_tenant, int max_blocks, int32_t* __restrict__ matched_len,
    int32_t* __restrict__ page_table, int32_t* __restrict__ path_end) {
  const int lane = threadIdx.x & (kWave - 1);
  const int r = blockIdx.x * kWavesPerWg + (threadIdx.x >> 6);
  if (r >= n_req) return;
  const int lo = uniform(req_off[r]), hi = uniform(req_off[r + 1]);
  const int tenant = uniform(req_tenant[r]);
  int nb = hi > lo ? (hi - lo) / SKV_BLOCK_TOKENS : 0;
  if (nb > max_blocks) nb = max_blocks;
  if (tenant < 0 || tenant >= t.n_tenants) nb = 0;
  const int32_t* x = req_tok + lo;
  int32_t* row = page_table + (size_t)r * max_blocks;   // holds block records during the walks, page ids at the end

  // One walk under the choices `ranks`: writes the matched blocks' record indices to row[], returns their
  // number; *n_choice / *counts describe the branch points met (how many visible copies each had).
  uint32_t limits = 0;   // SKV_LIMIT_* bits this request ran into (uniform)
  auto walk = [&](uint64_t ranks, int* n_choice, uint64_t* counts) {
    int j = 0, node = 0, dp = 0;
    uint64_t cnt = 0;
    bool stop = false;
    while (j < nb && !stop) {
      SkvNode cur = t.nodes[node];
      cur.tab_off = uniform(cur.tab_off);
      cur.tab_cap = uniform(cur.tab_cap);
      int n = 0;
      const int want = dp < kMaxChoice ? (int)((ranks >> (6 * dp)) & 63) : 0;
      const int child = find_child_ranked(t, cur, x + (size_t)j * 16, tenant, lane, want, &n, &limits);
      if (child < 0) break;
      if (n >= 2) {
        if (dp < kMaxChoice) {
          cnt |= (uint64_t)(n - 1) << (6 * dp);   // highest rank at this branch point
          ++dp;
        } else {
          limits |= SKV_LIMIT_BRANCH_POINTS;
        }
      }
      SkvNode nd = t.nodes[child];
      const int first = uniform(nd.first);
      const int nblk = uniform(nd.n_blocks);
      const int span = min(nblk, nb - j);
      for (int c = 0; c < span && !stop; c += kStepBlocks) {
        const int cb = min(kStepBlocks, span - c);
        const int ntok = cb * 16;
        const int32_t* tt = t.tok + (size_t)(first + c) * 16;
        const int32_t* xx = x + (size_t)j * 16;
        tok4 a[kSub], b[kSub];
        const tok4 z = {0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < kSub; ++u) {
          const int i = u * kWave + lane;    // vector index: tokens 4 i .. 4 i + 3, block i / 4
          a[u] = 4 * i < ntok ? ((const tok4*)xx)[i] : z;
          b[u] = 4 * i < ntok ? ((const tok4*)tt)[i] : z;
        }
        const int m = lane < cb ? t.meta[first + c + lane] : 0;
        int n_eq = cb;
#pragma unroll
        for (int u = kSub - 1; u >= 0; --u) {
          const uint64_t ne = ballot64(differ(a[u], b[u]));
          if (ne) n_eq = u * 16 + (__builtin_ctzll(ne) >> 2);
        }
        const uint64_t hidden = ballot64(m < 0 && (m & 0x7fffffff) != tenant);
        const int n_vis = hidden ? __builtin_ctzll(hidden) : cb;
        const int take = min(n_eq, n_vis);
        if (lane < take) row[j + lane] = first + c + lane;
        j += take;
        if (take < cb) stop = true;
      }
      node = child;
    }
    *n_choice = dp;
    *counts = cnt;
    return j;
  };

  uint64_t ranks = 0, best_ranks = 0;
  int best = -1;
  for (int walks = 0;; ++walks) {
    if (walks == kMaxWalks) { limits |= SKV_LIMIT_WALKS; break; }
    int dp = 0;
    uint64_t top = 0;
    const int len = walk(ranks, &dp, &top);
    if (len > best) { best = len; best_ranks = ranks; }
    if (len == nb) break;
    int i = dp - 1;   // deepest branch point that still has an untried copy
    while (i >= 0 && ((ranks >> (6 * i)) & 63) >= ((top >> (6 * i)) & 63)) --i;
    if (i < 0) break;
    const uint64_t keep = ((uint64_t)1 << (6 * i)) - 1;
    ranks = (ranks & keep) | ((((ranks >> (6 * i)) & 63) + 1) << (6 * i));
  }
  if (best < 0) best = 0;
  if (ranks != best_ranks) {   // row[] holds another walk: redo the chosen one
    int dp;
    uint64_t top;
    walk(best_ranks, &dp, &top);
  }
  __threadfence();   // row[] was written by other lanes of this wavefront: make the stores visible to the loads below
  const uint32_t tbit = 1u << (tenant & 31);
  const int tword = 1 + (tenant >> 5);
  const int last = best > 0 ? uniform(row[best - 1]) : -1;   // record of the last block on the chosen path
  for (int i = lane; i < best; i += kWave) {
    const int blk = row[i];
    row[i] = t.page[blk];
    uint32_t* ctr = t.ctr + (size_t)blk * SKV_CTR_STRIDE;
    atomicAdd(ctr, 1u);
    atomicOr(ctr + tword, tbit);
    t.epoch[blk] = t.cur_epoch;
  }
  if (lane == 0) matched_len[r] = best * SKV_BLOCK_TOKENS;
  if (lane == 0 && path_end) path_end[r] = last;
  if (lane == 0 && limits) atomicOr(t.limits, limits);
  for (int i = best + lane; i < max_blocks; i += kWave) row[i] = -1;
}

__global__ void skv_suffix_offsets_kernel(int n_req, const int32_t* __restrict__ req_off,
                                          const int32_t* __restrict__ matched_len,
                                          int32_t* __restrict__ q_off) {
  // one workgroup; chunked inclusive scan with a running carry
  __shared__ int32_t sh[1024];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) { carry = 0; q_off[0] = 0; }
  __syncthreads();
  for (int base = 0; base < n_req; base += 1024) {
    const int r = base + threadIdx.x;
    int v = 0;
    if (r < n_req) {
      v = req_off[r + 1] - req_off[r] - matched_len[r];
      if (v < 0) v = 0;
    }
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      int add = threadIdx.x >= o ? sh[threadIdx.x - o] : 0;
      __syncthreads();
      sh[threadIdx.x] += add;
      __syncthreads();
    }
    if (r < n_req) q_off[r + 1] = carry + sh[threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 0) carry += sh[1023];
    __syncthreads();
  }
}

}  // namespace

extern "C" int skv_match(skv_tree* t, int32_t n_req, const int32_t* d_req_off,
                         const int32_t* d_req_tokens, const int32_t* d_req_tenant, int32_t max_blocks,
                         int32_t* d_matched_len, int32_t* d_page_table, int32_t* d_path_end, void* stream) {
  if (!t || n_req < 0 || max_blocks < 0) return SKV_EINVAL;
  if (n_req == 0) return SKV_OK;
  if (!d_req_off || !d_req_tokens || !d_req_tenant || !d_matched_len) return SKV_EINVAL;
  if (max_blocks > 0 && !d_page_table) return SKV_EINVAL;
  const int grid = (n_req + kWavesPerWg - 1) / kWavesPerWg;
  if (t->has_copies)
    skv_match_copies_kernel<<<grid, kWave * kWavesPerWg, 0, (hipStream_t)stream>>>(
        t->dev, n_req, d_req_off, d_req_tokens, d_req_tenant, max_blocks, d_matched_len, d_page_table, d_path_end);
  else if (n_req <= kCoopMaxRequests)   // few requests: a workgroup each
    skv_match_kernel<kWavesPerWg><<<n_req, kWave * kWavesPerWg, 0, (hipStream_t)stream>>>(
        t->dev, n_req, d_req_off, d_req_tokens, d_req_tenant, max_blocks, d_matched_len, d_page_table, d_path_end);
  else
    skv_match_kernel<1><<<grid, kWave * kWavesPerWg, 0, (hipStream_t)stream>>>(
        t->dev, n_req, d_req_off, d_req_tokens, d_req_tenant, max_blocks, d_matched_len, d_page_table, d_path_end);
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_match_limits_read(skv_tree* t, uint32_t* limits_hit, int32_t clear, void* stream) {
  if (!t || !limits_hit) return SKV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  uint32_t v = 0;
  SKV_HIP(hipMemcpyAsync(&v, t->dev.limits, sizeof(v), hipMemcpyDeviceToHost, st));
  SKV_HIP(hipStreamSynchronize(st));
  if (clear && v) {
    const uint32_t zero = 0;
    SKV_HIP(hipMemcpyAsync(t->dev.limits, &zero, sizeof(zero), hipMemcpyHostToDevice, st));
    SKV_HIP(hipStreamSynchronize(st));
  }
  *limits_hit = v;
  return SKV_OK;
}

extern "C" int skv_suffix_offsets(int32_t n_req, const int32_t* d_req_off, const int32_t* d_matched_len,
                                  int32_t* d_q_off, void* stream) {
  if (n_req < 0 || !d_q_off) return SKV_EINVAL;
  if (n_req > 0 && (!d_req_off || !d_matched_len)) return SKV_EINVAL;
  skv_suffix_offsets_kernel<<<1, 1024, 0, (hipStream_t)stream>>>(n_req, d_req_off, d_matched_len, d_q_off);
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}
