/*
 * skv.h -- C ABI of the selective-reuse prefill path for AMD MI355X (gfx950).
 *
 * The path follows the SafeKV paper's request path (Section 4.1, "System Overview"):
 * a prefix lookup in the unified radix-tree index with a per-entry visibility check
 * (Section 4.3.1), the access-monitor update that feeds the RDR safeguard
 * (Section 4.2.2), reading the reused KV blocks through the entry's address vector
 * (Section 4.3.2, "Path Compression"), and prefill attention that reuses cached K/V
 * and computes only the uncached part (Section 2.1).
 *
 * Conventions
 *  - Pointers named d_* are DEVICE pointers (HIP device memory of the current device);
 *    all other pointers are HOST pointers.  `stream` is a hipStream_t passed as void*
 *    (NULL = the default stream).
 *  - The library never allocates or frees device memory.  Every device buffer, including
 *    the tree slab and the attention workspace, belongs to the caller and must stay valid
 *    until the work enqueued on `stream` has finished.
 *  - Calls only enqueue work on `stream` and return; they do not synchronise, except the
 *    host-driven structure changes skv_tree_build, skv_tree_insert, skv_evict and skv_tree_compact, which
 *    return after their uploads have completed, and skv_match_limits_read, which returns a host value.
 *  - Every function returns SKV_OK (0) or a negative error code; nothing is enqueued when
 *    an error is returned.  Arguments that live on the device (offsets, tenants, page ids)
 *    cannot be validated by the host: kernels clamp or skip values that are out of range
 *    instead of faulting, as described per function.
 *  - A tree handle is thread-compatible, not thread-safe: concurrent calls on one tree,
 *    or overlapping skv_match batches on different streams, race on the counters.
 *  - A KV block is 16 tokens.  KV pools are [n_pages][16][n_kv_heads][head_dim], row major.
 */
#ifndef SKV_H
#define SKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SKV_OK 0
#define SKV_EINVAL (-1) /* null pointer, malformed description, unsupported shape   */
#define SKV_ENOMEM (-2) /* caller-provided slab / workspace too small                */
#define SKV_ERANGE (-3) /* a value exceeds a built-in limit (e.g. n_tenants > 128)   */
#define SKV_EHIP (-4)   /* a HIP runtime call failed (see skv_last_hip_error)        */

#define SKV_BLOCK_TOKENS 16
#define SKV_MAX_TENANTS 128

#define SKV_F32 0
#define SKV_BF16 1

const char* skv_strerror(int code);
/* hipError_t of the last failing HIP call on this thread (0 if none). */
int skv_last_hip_error(void);

typedef struct skv_tree skv_tree; /* opaque host handle; owns host bookkeeping only */

/* Cached side: n_seq token sequences, each a whole number of 16-token blocks, with one
 * (private_tag, creator_id, KV address) triple per block (Section 4.3.1: every entry
 * stores private_tag and creator_id).  Per-block arrays are indexed by the block's
 * position in the concatenation of all sequences (its "input block id"). */
typedef struct {
  int32_t block_tokens;         /* must be 16 */
  int32_t n_tenants;            /* 1 .. 128 */
  int32_t n_pages;              /* pages in the KV pool; page ids lie in [0, n_pages) */
  int64_t n_seq;
  const int64_t* seq_off;       /* host [n_seq+1] token offsets, non-decreasing, multiples of 16 */
  const int32_t* tokens;        /* host [seq_off[n_seq]] */
  const uint8_t* blk_sensitive; /* host, per input block: 1 = private, 0 = shareable */
  const int32_t* blk_owner;     /* host, per input block: creator tenant in [0, n_tenants) */
  const int32_t* blk_page;      /* host, per input block: page id */
} skv_tree_desc;

/* Upper bound, in bytes, of the device slab skv_tree_build needs for this description. */
int skv_tree_build_size(const skv_tree_desc* desc, size_t* device_bytes);

/* Bytes of a slab that can hold block_capacity blocks (described plus later inserted ones, repeats
 * included).  SKV_ERANGE beyond 2^26 - 1 blocks. */
int skv_tree_size_for_capacity(int64_t block_capacity, size_t* device_bytes);

/* Build the index (Section 4.3.1 Insert; Section 4.3.2 path compression): inserts the
 * sequences in order, where a block whose whole block-prefix is already cached keeps the
 * first insertion's metadata and page; collapses every non-branching run of blocks into one
 * node carrying a per-block page-id vector; writes the flattened tree into d_slab (256-byte
 * aligned, at least skv_tree_build_size bytes) and zeroes the counters.  A larger slab leaves room
 * for skv_tree_insert: the capacity is the largest block count whose layout fits into `bytes`.
 * Errors: SKV_EINVAL for null pointers, block_tokens != 16, offsets that decrease or are not
 * multiples of 16, an owner outside [0, n_tenants), a page id outside [0, n_pages), the same
 * page id on two distinct cached blocks, or a misaligned slab; SKV_ERANGE for n_tenants
 * outside [1, 128] or more than 2^31-1 blocks; SKV_ENOMEM if `bytes` is too small.
 * Synchronises `stream` before returning. */
int skv_tree_build(const skv_tree_desc* desc, void* d_slab, size_t bytes, void* stream,
                   skv_tree** out);

/* Insert after a prefill (Section 4.3.1 Insert: new KV blocks are appended along the request's path;
 * Section 4.1 and Section 6: every new block starts private, with the requester as creator_id).  All arrays are HOST
 * arrays.  For request r (tokens req_tokens[req_off[r] .. req_off[r+1]), tenant req_tenant[r]) the full
 * 16-token blocks that the tree does not hold yet are appended below the point where the request's token
 * path leaves the tree (splitting a compressed node when that point lies inside it), private to the tenant.
 * The index keeps one entry per block-prefix: blocks whose tokens are already on the path keep their entry,
 * whoever created it, so a tenant that is blocked by another tenant's private block adds only what lies
 * beyond the cached path.  new_pages[r*max_new_blocks + j] is the pool page of the request's block
 * matched_len[r]/16 + j (the table skv_scatter_kv wrote through; matched_len as skv_match returned it);
 * insertion stops at the first block without a page (< 0, or j >= max_new_blocks).  Requests are inserted
 * in order, so a later request of the batch finds what an earlier one added.
 * private_copies != 0 (Section 4.1: selective isolation leaves redundant copies): a requester stopped by an
 * entry it may not see adds its own copy.  The request's longest visible path is looked up in the tree as
 * it stands, and all full blocks beyond that path are appended below its end, private to the tenant, next
 * to whatever other tenants cached there.  A position may then hold several children that start with the
 * same block; from the first such insertion on skv_match follows every copy whose first block the tenant
 * may see and returns the longest path (equally long ones: the path through the copy with the smaller
 * input block id at the first difference).  Its search explores at most 10 such branch points per request
 * exhaustively, the 64 oldest visible copies per position and 4096 root-to-end walks; a request that runs into one
 * of these limits may be given a shorter path than the longest one, and the limit is recorded (skv_match_limits_read).
 * path_end (HOST, n_req entries, may be NULL; used with private_copies only): the path ends skv_match wrote for
 * this batch (copied to the host by the caller), taken on the tree and the visibility bits as they are when the
 * insert is called.  The lookup has then already found each requester's longest visible path, and the insert only
 * continues it through blocks that earlier requests of the same batch added for the same tenant (nothing else can
 * have become visible to that tenant in between) -- no search and no visibility bits are needed.  matched_len[r]
 * must be the matched length of the same lookup.  Without path_end the insert searches itself, on the host, against
 * the tree as earlier requests of the batch left it; it then uses the host's copy of the visibility bits, which is
 * fetched from the device again (on `stream`) only if skv_promote or skv_window_roll has been enqueued since it
 * was taken.
 * New entries receive the input
 * block ids n_in_blocks, n_in_blocks + 1, ... in that order, start with zeroed counters, and are visible to
 * skv_match calls enqueued afterwards.  first_inserted[r] / n_inserted[r] report the index of the request's
 * first new block and their number (pages given for blocks below first_inserted[r] stay unused).
 * Errors, nothing changed: SKV_EINVAL for null pointers, decreasing offsets, a tenant outside
 * [0, n_tenants), a page id outside [0, n_pages), already backing a cached block, or named twice, or a path end
 * that does not fit the request (no such record, an evicted one, or not the request's block matched_len/16 - 1);
 * SKV_ENOMEM when the slab's capacity (blocks, or child-table slots) would be exceeded (records that evictions
 * left behind count until skv_tree_compact reclaims them).
 * Copies the changed records to the device on `stream` and synchronises it before returning.  Must not
 * overlap with other calls on the tree. */
int skv_tree_insert(skv_tree* tree, int32_t n_req, const int32_t* req_off, const int32_t* req_tokens,
                    const int32_t* req_tenant, const int32_t* matched_len, const int32_t* new_pages,
                    int32_t max_new_blocks, int32_t private_copies, const int32_t* path_end, int32_t* first_inserted,
                    int32_t* n_inserted, void* stream);

/* Global epoch counter (Section 4.3.2: the index keeps a global epoch_counter and every entry its most
 * recent access epoch).  skv_match calls enqueued after this call stamp `epoch` on every block they match;
 * skv_tree_insert stamps it on the blocks it adds.  Blocks of the initial build start at epoch 0. */
int skv_set_epoch(skv_tree* tree, uint32_t epoch);

/* Last access epoch per input block id (device array of n_in_blocks entries; 0 for blocks without entry). */
int skv_block_epochs_read(skv_tree* tree, uint32_t* d_epoch, void* stream);

/* Eviction (Section 4.3.1 Evict: epoch-based LRU, entries in use are protected; Section 4.3.2 progressive
 * eviction: space is reclaimed from leaf to root, and a compressed chain releases the entries of its
 * address vector one by one from its far end, the node itself only when the vector is empty).  Only the
 * last block of a childless node can be removed without cutting off other entries.  Among these candidates,
 * skipping the ones whose input block id is listed in protect_ids (HOST array: blocks in use, e.g. those a
 * running batch matched), the block with the oldest access epoch is removed first (ties: the smaller input
 * block id); this repeats until n_want blocks are gone or no candidate is left.  evicted_ids / evicted_pages
 * (HOST arrays of n_want entries) receive the removed blocks and their pool pages in removal order, so the
 * caller can hand the pages out again; *n_evicted their number.  Removed blocks read as absent from then on
 * (skv_counters_read and skv_block_state_read report them like blocks without entry); their record space in
 * the slab is reused after skv_tree_compact.  Reads the epochs back from the device and uploads the changed records on
 * `stream`, synchronising it; must not overlap with other calls on the tree.
 * Errors: SKV_EINVAL for null pointers or negative counts. */
int skv_evict(skv_tree* tree, int64_t n_want, const int32_t* protect_ids, int64_t n_protect,
              int32_t* evicted_ids, int32_t* evicted_pages, int64_t* n_evicted, void* stream);

/* Reclaim the record space that evictions and insertions leave behind (Section 4.3.2 Progressive Eviction: a
 * compressed chain's address vector shrinks as its entries are released, and the chain is removed once it is
 * empty): evicted block records, emptied nodes, abandoned child tables.  The live structure is laid out afresh in
 * the same slab, and the input block ids are renumbered densely in their old order: id_map (HOST, one entry per
 * input block id before the call) receives each id's new value, -1 for blocks that no longer exist;
 * *n_in_blocks_after (may be NULL) the new id count.  Lookups, counters, visibility bits and epochs are unchanged
 * apart from the renumbering; the capacity left for skv_tree_insert is the slab's capacity minus the live blocks.
 * Reads the kernels' per-block state back, uploads the whole structure on `stream` and synchronises it; must not
 * overlap with other calls on the tree.  Errors: SKV_EINVAL for a null tree or map. */
int skv_tree_compact(skv_tree* tree, int32_t* id_map, int64_t* n_in_blocks_after, void* stream);

/* n_nodes: compressed nodes (root excluded); n_blocks: distinct cached blocks (evicted ones not counted);
 * n_in_blocks: blocks in the description (repeats included).  Any pointer may be NULL. */
int skv_tree_info(const skv_tree* tree, int64_t* n_nodes, int64_t* n_blocks, int64_t* n_in_blocks);

/* Frees the host handle.  The slab stays the caller's. */
void skv_tree_destroy(skv_tree* tree);

/* Longest visible prefix match + access-monitor update (Section 4.3.1 Search, Section 4.2.2).
 * For request r with tokens d_req_tokens[d_req_off[r] .. d_req_off[r+1]) and tenant
 * d_req_tenant[r]: k_r = the largest k <= min(floor(N_r/16), max_blocks) such that the first
 * k blocks follow a root path of the tree and each of them is shareable or created by that
 * tenant (the walk stops at the first block that is absent or not visible).
 * Writes d_matched_len[r] = 16*k_r and d_page_table[r*max_blocks + j] = page id of block j for
 * j < k_r, -1 for k_r <= j < max_blocks.  For every matched block adds 1 to its hit counter
 * and records the tenant in its distinct-tenant set (commutative atomics: the batch result
 * does not depend on execution order), and stamps the block with the current epoch (skv_set_epoch).
 * On a tree that holds per-tenant copies (skv_tree_insert with private_copies) a position can offer several
 * children that start with the request's next block; the walk then follows every copy whose first block the
 * tenant may see and the longest path wins, as described at skv_tree_insert; only that path's blocks are
 * counted and stamped.
 * A request whose tenant is outside [0, n_tenants) or whose offsets decrease matches nothing.
 * d_path_end (DEVICE, n_req entries, may be NULL) receives where each request's path ends inside the index: the
 * record number of its last matched block, -1 if nothing matched.  The number is meaningful only to
 * skv_tree_insert, which can then append a request's new blocks below that point without looking the path up
 * again; it stays valid until the next skv_evict or skv_tree_compact.
 * Errors: SKV_EINVAL for null pointers or negative sizes.  n_req == 0 is a no-op. */
int skv_match(skv_tree* tree, int32_t n_req, const int32_t* d_req_off, const int32_t* d_req_tokens,
              const int32_t* d_req_tenant, int32_t max_blocks, int32_t* d_matched_len,
              int32_t* d_page_table, int32_t* d_path_end, void* stream);

/* Limits of the branching lookup (trees with per-tenant copies, Section 4.1): which of them any request has run
 * into since the tree was built or the word was last cleared -- SKV_LIMIT_BRANCH_POINTS (more than 10 positions
 * with several visible copies on one walk), SKV_LIMIT_COPIES (more than 64 visible copies at one position),
 * SKV_LIMIT_WALKS (more than 4096 walks for one request).  0 means every result so far is the longest visible
 * path.  limits_hit is a HOST word; clear != 0 resets the record.  Synchronises `stream`. */
#define SKV_LIMIT_BRANCH_POINTS 1u
#define SKV_LIMIT_COPIES 2u
#define SKV_LIMIT_WALKS 4u
int skv_match_limits_read(skv_tree* tree, uint32_t* limits_hit, int32_t clear, void* stream);

/* Current-window counters per input block id (Section 4.2.2: hit_cur and u_cnt;
 * RDR = u_cnt / hit_cur): d_hit[b] = hits, d_ucnt[b] = distinct tenants.  Both arrays have
 * n_in_blocks entries; blocks that repeat an already cached block-prefix read 0. */
int skv_counters_read(skv_tree* tree, uint32_t* d_hit, uint32_t* d_ucnt, void* stream);

/* Clear the current window (Section 4.2.2: the access monitor keeps its counters over a rolling window):
 * zero every block's hit counter and tenant set; previous-window counters and the predicate streak are kept. */
int skv_counters_reset(skv_tree* tree, void* stream);

/* Safeguard policy (Section 4.2.2 and Section 6).  RDR = u_cnt / hit_cur is compared with
 * tau = tau_num / tau_den as an exact rational (integers only).  direction 0: the predicate holds when
 * RDR < tau (Section 6: probing lowers the RDR); direction 1: when RDR > tau and the previous window's
 * distinct-tenant count u_pre <= u_pre_max (Section 4.2.2: narrow history, dispersed present).  Blocks
 * with hit_cur == 0 or hit_cur < min_hits never meet it.  The paper fixes neither the direction nor the
 * threshold, so both are the caller's. */
typedef struct {
  int32_t direction;   /* 0 or 1 */
  uint32_t tau_num, tau_den; /* tau_den >= 1 */
  uint32_t min_hits;
  uint32_t n_consec;   /* >= 1: consecutive windows the predicate must hold before demotion */
  uint32_t u_pre_max;  /* used by direction 1 only */
} skv_rdr_policy;

/* Safeguard step at a window boundary, over every cached block: evaluate the predicate on the current
 * window's counters; a shareable block whose predicate has now held for n_consec consecutive windows is
 * demoted to private (from then on only its creator_id matches it -- Section 6: after demotion, future
 * cross-tenant hits on that block stop); then roll the window (hit_pre <- hit_cur, u_pre <- u_cnt, current
 * counters and tenant set cleared).  If d_n_demoted is not NULL it receives the number of blocks demoted.
 * Must not overlap with skv_match on the same tree.  Errors: SKV_EINVAL for null tree / policy,
 * direction outside {0,1}, tau_den == 0 or n_consec == 0. */
int skv_window_roll(skv_tree* tree, const skv_rdr_policy* policy, int32_t* d_n_demoted, void* stream);

/* Promotion (Section 4.2.3: once background verification marks a block shareable, its visibility bit is
 * flipped so that later lookups may reuse it across tenants): clears private_tag of the entries created by
 * the n input block ids in d_block_ids (device, int32).  Ids outside [0, n_in_blocks) and ids of blocks
 * that repeat an already cached block-prefix are ignored.  Must not overlap with skv_match on the tree. */
int skv_promote(skv_tree* tree, const int32_t* d_block_ids, int32_t n, void* stream);

/* Per input block id: private_tag (0 shareable, 1 private, 255 for a block that repeats an already cached
 * block-prefix) and the previous window's counters (Section 4.2.2: hit_pre, u_pre).  Arrays of n_in_blocks
 * entries; any of them may be NULL. */
int skv_block_state_read(skv_tree* tree, uint8_t* d_private, uint32_t* d_hit_pre, uint32_t* d_u_pre,
                         void* stream);

/* Device-side layout of the uncached suffixes: S_r = N_r - matched_len[r];
 * d_q_off[0] = 0, d_q_off[r+1] = d_q_off[r] + S_r  ([n_req+1], row offsets into Q/K_new/V_new/O). */
int skv_suffix_offsets(int32_t n_req, const int32_t* d_req_off, const int32_t* d_matched_len,
                       int32_t* d_q_off, void* stream);

typedef struct {
  int32_t n_q_heads;
  int32_t n_kv_heads; /* divides n_q_heads; query head h uses kv head h / (n_q_heads/n_kv_heads) */
  int32_t head_dim;   /* SKV_BF16: 128;  SKV_F32: 64 or 128 */
  int32_t dtype;      /* SKV_F32 or SKV_BF16: type of Q, K, V, the pools and the output */
  float scale;        /* softmax scale; a value <= 0 (or not finite) selects 1/sqrt(head_dim), the scaled
                         dot-product attention of Section 2.1 */
} skv_attn_desc;

/* Gather the reused pages (Section 4.3.2: the lookup reads the required KV blocks directly from
 * the address vector): request r's k_r matched K pages are copied, in order, to
 * d_kctx[ctx_off[r] .. ctx_off[r] + 16*k_r) (token rows of n_kv_heads*head_dim elements), same
 * for V, with ctx_off the exclusive prefix sum of matched_len, which is also written to
 * d_ctx_off ([n_req+1], int64).  Byte-exact copy.  Pages whose id is outside [0, n_pages) and
 * rows at or beyond ctx_capacity_tokens are skipped.
 * Errors: SKV_EINVAL for null pointers, unsupported dtype, or a page size that is not a multiple
 * of 16 bytes. */
int skv_gather_kv(const skv_attn_desc* desc, int32_t n_req, const void* d_kpool, const void* d_vpool,
                  int32_t n_pages, const int32_t* d_matched_len, const int32_t* d_page_table,
                  int32_t max_blocks, int64_t* d_ctx_off, void* d_kctx, void* d_vctx,
                  int64_t ctx_capacity_tokens, void* stream);

/* Insert side of the KV pool (Section 4.3.1 Insert: newly generated KV blocks are appended to the cache):
 * the full 16-token blocks of request r's uncached suffix (rows d_q_off[r] + 16 j .. + 15 of d_knew / d_vnew)
 * are written to pool page d_new_pages[r*max_new_blocks + j]; entries that are negative, outside
 * [0, n_pages), or beyond the suffix's floor(S_r / 16) full blocks are skipped.  Byte-exact copy, the inverse
 * of skv_gather_kv.  Two entries naming the same page race.  Errors as skv_gather_kv. */
int skv_scatter_kv(const skv_attn_desc* desc, int32_t n_req, const void* d_knew, const void* d_vnew,
                   const int32_t* d_q_off, const int32_t* d_new_pages, int32_t max_new_blocks, void* d_kpool,
                   void* d_vpool, int32_t n_pages, void* stream);

/* Plain device-to-device streaming copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned, the
 * ranges must not overlap), with the same vector width and access shape as the page copies of skv_gather_kv and
 * skv_scatter_kv but no page table.  It is the copy of known size that HBM traffic counters are scaled by, and
 * its rate is the box's own copy ceiling that the gather (Section 4.3.2) is compared with.
 * Errors: SKV_EINVAL for null or misaligned pointers or a size that is not a multiple of 16. */
int skv_stream_copy(void* d_dst, const void* d_src, size_t bytes, void* stream);

/* Measurement aid for the attention roofline (Section 2.1 attention; Section 6 reports prefill time): the rate at
 * which the chip sustains the bf16 matrix instruction of skv_prefill_attn (32x32x16, fp32 accumulate) on operand
 * values of the caller's choosing, with nothing else running -- operands stay in registers, one workgroup of eight
 * wavefronts per compute unit, `iters` rounds of 16 instructions each.  The clock under matrix load depends on the operand values,
 * so the rate for values distributed like a workload's K/V/Q is the ceiling that workload's attention can be held
 * against; constants give the nominal peak.  d_operands: DEVICE, at least SKV_MFMA_RATE_OPERAND_BYTES bytes of
 * bf16 values, 16-byte aligned (read once); d_sink: DEVICE, at least SKV_MFMA_RATE_SINK_BYTES bytes (overwritten,
 * keeps the results alive).  *flops (HOST, may be NULL) receives the floating-point operations one call issues;
 * the caller times the call on `stream`.  side_work: 0 = the matrix instruction alone; 1 = every matrix
 * instruction accompanied by what the softmax of skv_prefill_attn issues per matrix instruction at the least (its A
 * operand read from LDS, one multiply-add, one exponential, one add, half a packed conversion) on values that
 * depend on no matrix result, with no global load and no barrier: the rate that instruction mix can reach at all.
 * Errors: SKV_EINVAL for null or misaligned pointers, iters < 1 or side_work other than 0 or 1; SKV_ENOMEM for
 * buffers that are too small. */
#define SKV_MFMA_RATE_OPERAND_BYTES ((size_t)512 * 512 * 6 * 32)
#define SKV_MFMA_RATE_SINK_BYTES ((size_t)512 * 512 * 4)
int skv_mfma_rate(const void* d_operands, size_t operand_bytes, int32_t iters, int32_t side_work, float* d_sink,
                  size_t sink_bytes, double* flops, void* stream);

/* Bytes of device workspace skv_prefill_attn needs for n_req requests and at most
 * total_q_rows uncached tokens in the batch (the work list of the bf16 kernel and one page of zeros that
 * stands in for key groups without data); the call overwrites it. */
int skv_prefill_attn_workspace_size(const skv_attn_desc* desc, int32_t n_req, int64_t total_q_rows,
                                    size_t* bytes);

/* Causal GQA prefill attention of the uncached suffixes (Section 2.1).  For request r, suffix
 * position i in [0, S_r), S_r = d_q_off[r+1] - d_q_off[r], query head h:
 *   O[q_off[r]+i, h] = softmax_j(scale * q[q_off[r]+i, h] . k_j) . v_j
 * over j in [0, L_r + i]: first the L_r = d_matched_len[r] reused positions (whole blocks: a value that is
 * not a multiple of 16 is rounded down, as in skv_gather_kv), read from the
 * pools through d_page_table[r*max_blocks + j/16] at slot j%16, then the request's own new
 * positions 0..i from d_knew / d_vnew (rows q_off[r] + (j - L_r)).
 * d_q, d_out: [total rows][n_q_heads][head_dim]; d_knew, d_vnew: [total rows][n_kv_heads][head_dim].
 * total_q_rows is a host-side upper bound of d_q_off[n_req] (the rows allocated in d_q / d_out);
 * rows beyond d_q_off[n_req] are left untouched.  S_r == 0 is legal.  Pages with an id outside
 * [0, n_pages) are read as zeros.  bf16 computes QK^T and PV on the matrix cores with fp32
 * accumulation and fp32 softmax; fp32 computes in fp32 throughout.
 * Errors: SKV_EINVAL for null pointers or unsupported shapes, SKV_ENOMEM if the workspace is
 * smaller than skv_prefill_attn_workspace_size. */
int skv_prefill_attn(const skv_attn_desc* desc, int32_t n_req, const void* d_q, const void* d_knew,
                     const void* d_vnew, const int32_t* d_q_off, int64_t total_q_rows,
                     const void* d_kpool, const void* d_vpool, int32_t n_pages,
                     const int32_t* d_matched_len, const int32_t* d_page_table, int32_t max_blocks,
                     void* d_out, void* d_workspace, size_t workspace_bytes, void* stream);

/* skv_prefill_attn for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * skv_prefill_attn without the workspace: the work list and the page of zeros live in a device array built
 * into the library (SKV_STATIC_SCRATCH_BYTES per GPU, held until the process ends), whose address on the
 * current device is looked up on the first call there.  The call allocates and frees nothing.
 * SKV_ERANGE when skv_prefill_attn_workspace_size for (n_req, total_q_rows) exceeds SKV_STATIC_SCRATCH_BYTES
 * (bf16 with 4 query heads per kv head: about 8 million uncached tokens per batch).
 * All calls on one GPU share the array, whichever stream they use: calls that overlap on a GPU race; calls
 * on one stream, or ordered by events, are safe (each call rewrites everything it reads). */
#define SKV_STATIC_SCRATCH_BYTES (4u << 20)
int skv_prefill_attn_static(const skv_attn_desc* desc, int32_t n_req, const void* d_q, const void* d_knew,
                            const void* d_vnew, const int32_t* d_q_off, int64_t total_q_rows,
                            const void* d_kpool, const void* d_vpool, int32_t n_pages,
                            const int32_t* d_matched_len, const int32_t* d_page_table, int32_t max_blocks,
                            void* d_out, void* stream);

/* Decode-step attention (Section 2.1: at every decode step the new token attends to the cached K/V of all
 * earlier tokens).  For request r, d_q holds one query row per query head ([n_req][n_q_heads][head_dim]) and
 * d_ctx_len[r] the number of cached tokens it attends to (the current token's K/V included, already written
 * to the pool); token j lives in page d_page_table[r*max_blocks + j/16], row j%16.
 * d_out[r][h] = sum_j softmax_j(scale * q[r][h] . K[j]) V[j] over j < ctx_len[r], kv head h / (n_q_heads /
 * n_kv_heads).  bf16, head_dim 128, at most 16 query heads per kv head (SKV_EINVAL otherwise).  ctx_len is
 * clamped to [0, 16*max_blocks]; a request with no cached token gets zeros; a page id outside [0, n_pages)
 * reads as zeros; rows of the last page beyond ctx_len are never used, whatever they hold.  Pools of several
 * layers are handled by passing the layer's base pointers.  The workspace (device, 16-byte aligned,
 * skv_decode_attn_workspace_size bytes) holds the partial softmax states of the key splits; it is overwritten
 * by every call.  Errors as skv_prefill_attn. */
int skv_decode_attn_workspace_size(const skv_attn_desc* desc, int32_t n_req, int32_t max_blocks, size_t* bytes);
int skv_decode_attn(const skv_attn_desc* desc, int32_t n_req, const void* d_q, const void* d_kpool,
                    const void* d_vpool, int32_t n_pages, const int32_t* d_ctx_len, const int32_t* d_page_table,
                    int32_t max_blocks, void* d_out, void* d_workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SKV_H */
