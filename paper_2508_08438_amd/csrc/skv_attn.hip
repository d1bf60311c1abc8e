// Causal GQA prefill attention of the uncached suffix over reused paged prefix KV plus the
// request's own new KV.
//
// SafeKV Section 2.1: inference attends over all previous tokens; with KV caching the K/V of
// the cached prefix are reused and only the new tokens' part is computed.  Row i of the
// suffix therefore attends to the L reused positions (read from the page pool through the
// page table the match produced) and to its own positions 0..i.
//
// bf16 path: flash-style streaming over 64-key tiles with online softmax in fp32; the two
// contractions (K.Q^T and V^T.P^T) run on the matrix cores (v_mfma_f32_32x32x16_bf16), the
// softmax on the vector ALU.  A workgroup of eight wavefronts shares every K/V tile through
// LDS; each wavefront owns 32 query rows of one head (the query heads of one kv head share a
// workgroup, so a K/V tile is fetched once for the group).  K/V rows travel global -> LDS with
// direct-to-LDS loads (no stop in registers, no LDS store instructions), three stages each.
// The products are formed transposed (S^T = K Q^T, O^T = V^T P^T) so that a query is a
// lane-column of the MFMA accumulator: row sums are register reductions, and the P^T
// accumulator registers are already in the B-operand layout of the second product; V^T
// fragments come from the LDS transpose load.  The inner loop is a three-stage software
// pipeline over 32-key sub-tiles: the scores of sub-tile h + 1, the softmax of sub-tile h and
// the output update with sub-tile h - 1 share a half-step, in which nothing depends on
// anything else, so MFMAs and vector instructions alternate in the instruction stream.
// fp32 path: one wavefront per output row, plain fp32 arithmetic (correctness configuration).
#include <atomic>

#include "skv_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kD = 128;          // head dim of the bf16 kernel
constexpr int kBN = 64;          // keys per LDS tile
constexpr int kKStages = 3;      // LDS stages of K: tiles kt, kt + 1 in use, kt + 2 arriving
constexpr int kVStages = 3;      // LDS stages of V: tiles kt - 1, kt in use, kt + 1 arriving
constexpr int kStageRows = 16;   // rows of a wave's Q / O staging tile
constexpr float kSumLimit = 4096.f;   // move the softmax reference when a lane's sum of 16 exponentials exceeds this
constexpr int kRowsPerWave = 32; // query rows per wavefront
constexpr int kWaves = 8;        // two per SIMD: one wave's softmax overlaps the other's MFMAs
constexpr int kThreads = kWaves * 64;
// LDS tile layout (K and V alike): a 64-key tile is 16 segments of 4 keys, 1040 bytes apart.  Inside a segment the
// 16-byte piece (key q of the segment, chunk c of the 256-byte row) sits at (c / 4) * 256 + q * 64 + (c % 4) * 16.
// One direct-to-LDS load of a wavefront fills one segment: the hardware puts what lane i fetched at byte 16 i, so
// lane i fetches chunk 4 (i / 16) + i % 4 of key (i / 4) % 4 -- four lanes read 64 consecutive bytes of a row.
// The K fragment reads (ds_read_b128: 16 lanes = 16 keys, one chunk) and the V^T fragment reads
// (ds_read_b64_tr_b16: 32 lanes = 4 keys x 64 bytes) are free of bank conflicts, and the addresses of different
// fragments differ by constants only.
constexpr int kSeg = 520;            // bf16 elements per segment (1040 B)
constexpr int kTile = 16 * kSeg;     // bf16 elements per 64-key tile
constexpr float kLog2e = 1.4426950408889634f;

struct AttnParams {
  const void *q, *knew, *vnew, *kpool, *vpool;
  void* out;
  const int32_t *q_off, *matched_len, *page_table;
  const int32_t* items;      // kItemInts ints per work item
  const int32_t* n_items;
  const char* zero_page;     // 16 rows of zeros: stands in for a group of keys that has no data
  int n_req, max_blocks, n_pages, Hq, Hkv;
  int heads_per_wg;          // query heads of one kv head handled by one workgroup (1, 2 or 4)
  float scale;
};

// ---- work list ---------------------------------------------------------------------------------
// One workgroup.  items[] lists one 32-byte record per (request, q tile) pair -- {request, first suffix row of
// the tile, first row of the request in Q, its suffix length S, its reused length L, end row of the tile} -- so
// that a workgroup of the attention kernel learns everything about its piece of work from one load.  A request's
// heaviest (last) tile first.  The q tiles of a request are cut so that L + (first row of a tile) is a multiple of the
// 64-key tile: the first tile is short when L is not, and every later tile ends exactly where a key tile ends, so
// no workgroup streams a key tile for the sake of a few keys of round-up -- unless the short first tile makes the
// request one tile longer than cutting from row 0 would and the reused prefix is long (L > S / 2): a tile more costs
// a pass over about L + S / 2 keys, the round-up one more 64-key iteration in each of the S / 64 tiles.
constexpr int kItemInts = 8;
__global__ void attn_schedule_kernel(int n_req, const int32_t* __restrict__ q_off,
                                     const int32_t* __restrict__ matched_len, int pos_per_wg,
                                     int max_items, int32_t* __restrict__ n_items, int32_t* __restrict__ items,
                                     uint4* __restrict__ zero_page, int zero_vec) {
  __shared__ int32_t sh[1024];
  for (int i = threadIdx.x; i < zero_vec; i += 1024) zero_page[i] = make_uint4(0u, 0u, 0u, 0u);
  __shared__ int32_t carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < n_req; base += 1024) {
    const int r = base + threadIdx.x;
    int nt = 0, S = 0, qb = 0, L = 0, head_rows = 0;   // head_rows: rows of the short first tile (0: none)
    if (r < n_req) {
      qb = q_off[r];
      S = q_off[r + 1] - qb;
      L = matched_len[r] > 0 ? matched_len[r] & ~(SKV_BLOCK_TOKENS - 1) : 0;   // whole blocks only
      head_rows = min(S, (kBN - L % kBN) % kBN);
      nt = S > 0 ? (head_rows > 0 ? 1 : 0) + (S - head_rows + pos_per_wg - 1) / pos_per_wg : 0;
      const int nt_plain = (S + pos_per_wg - 1) / pos_per_wg;
      if (nt_plain < nt && 2 * L > S) {   // the short first tile would cost a whole extra tile: cut from row 0 instead
        head_rows = 0;
        nt = nt_plain;
      }
    }
    sh[threadIdx.x] = nt;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      int add = threadIdx.x >= o ? sh[threadIdx.x - o] : 0;
      __syncthreads();
      sh[threadIdx.x] += add;
      __syncthreads();
    }
    const int start = carry + sh[threadIdx.x] - nt;
    for (int k = 0; k < nt; ++k) {
      if (start + k < max_items) {
        int4* rec = (int4*)(items + (size_t)kItemInts * (start + k));
        const int j = nt - 1 - k;   // tile index within the request
        int row0, row1;
        if (head_rows > 0 && j == 0) {
          row0 = 0;
          row1 = head_rows;
        } else {
          row0 = head_rows + (j - (head_rows > 0 ? 1 : 0)) * pos_per_wg;
          row1 = min(S, row0 + pos_per_wg);
        }
        rec[0] = make_int4(r, row0, qb, S);
        rec[1] = make_int4(L, row1, 0, 0);

      }
    }
    __syncthreads();
    if (threadIdx.x == 0) carry += sh[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0) *n_items = carry < max_items ? carry : max_items;
}

// ---- bf16 MFMA kernel --------------------------------------------------------------------------
// Value of the lane 32 positions away (the other half of the wavefront): v_permlane32_swap exchanges the
// upper half of its first operand with the lower half of its second.
__device__ inline float swap_halves(float x) {
  float a = x, b = x;
  // the wait states the compiler places between a VALU write and this instruction are added by hand
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return (threadIdx.x & 32) ? a : b;
}
// max / sum of a value and the one 32 lanes away: after the swap `a` holds the lower half's value in both halves
// and `b` the upper half's, so no lane select is needed
__device__ inline float max_halves(float x) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return fmaxf(a, b);
}

// LDS fragment reads as inline assembly, with their waits placed by hand.  The compiler puts a full
// s_waitcnt vmcnt(0) in front of LDS reads it cannot tell apart from the targets of the direct-to-LDS loads in
// flight, which would stall every tile on the copies of the next one; the tile barrier already orders those
// copies against the reads.  The LDS returns data in issue order, so "at most n operations outstanding" means that
// everything issued before the n youngest reads has arrived.  A wait takes the registers it guards as in/out
// operands: their consumers then depend on it and cannot be moved in front of it.
__device__ __forceinline__ uint32_t lds_addr(const void* ptr) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)ptr;
}
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr, int byte_off) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "i"(byte_off));
  return v;
}
__device__ __forceinline__ s16x4 lds_read_tr16_b64(uint32_t addr, int byte_off) {
  s16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "i"(byte_off));
  return v;
}
__device__ __forceinline__ void lds_wait(int n, bf16x8& a) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "i"(n));
}
__device__ __forceinline__ void lds_wait(int n, bf16x8& a, bf16x8& b, bf16x8& c, bf16x8& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "i"(n));
}

__global__ __launch_bounds__(kThreads, 2) void attn_bf16_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) __bf16 smem[kKStages * kTile + kVStages * kTile +
                                                      kWaves * kStageRows * kD];
  __bf16* const Ks = smem;
  __bf16* const Vs = smem + kKStages * kTile;
  // [kWaves][16 rows][16 chunks of 8 bf16]: each wave's own staging tile for its Q rows on the way in and its O rows
  // on the way out (16 rows at a time), 16-byte chunks XOR-swizzled by row so that row-wise and fragment-wise
  // accesses are conflict free
  __bf16* const stage = Vs + kVStages * kTile + (threadIdx.x >> 6) * (kStageRows * kD);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
  const int l32 = lane & 31;
  const int half = lane >> 5;

  // ---- which piece of work: XCD-aware decode (workgroup b runs on XCD b % 8) ----
  const int G = p.Hq / p.Hkv;
  const int n_hg = G / p.heads_per_wg;               // head groups per kv head
  int item, kvh, hg;
  {
    const int b = blockIdx.x;
    if (p.Hkv % 8 == 0) {
      // all work of one kv head stays on one XCD, so its K/V tiles are re-read from that XCD's L2
      const int per = p.Hkv / 8;
      const int xcd = b & 7, slot = b >> 3;
      kvh = xcd + 8 * (slot % per);
      const int rest = slot / per;
      hg = rest % n_hg;
      item = rest / n_hg;
    } else {
      kvh = b % p.Hkv;
      const int rest = b / p.Hkv;
      hg = rest % n_hg;
      item = rest / n_hg;
    }
  }
  // the record is read together with the item count (the grid bound keeps the index inside the list)
  const int4 rec0 = ((const int4*)(p.items + (size_t)kItemInts * item))[0];
  const int L = __builtin_amdgcn_readfirstlane(p.items[(size_t)kItemInts * item + 4]);
  const int row1 = __builtin_amdgcn_readfirstlane(p.items[(size_t)kItemInts * item + 5]);   // end row of the q tile
  if (item >= *p.n_items) return;
  const int r = __builtin_amdgcn_readfirstlane(rec0.x);
  const int row0 = __builtin_amdgcn_readfirstlane(rec0.y);                                  // first row of the q tile
  const int qbase = __builtin_amdgcn_readfirstlane(rec0.z);
  const int S = __builtin_amdgcn_readfirstlane(rec0.w);
  const int Ltot = L + S;

  const int head = kvh * G + hg * p.heads_per_wg + (wave % p.heads_per_wg);
  const int pos0 = row0 + (wave / p.heads_per_wg) * kRowsPerWave;             // first row of this wave
  const int n_tiles = (L + row1 + kBN - 1) / kBN;                             // 64-key tiles the workgroup streams
  const int wave_key_end = pos0 < row1 ? L + min(row1, pos0 + kRowsPerWave) : 0;  // this wave needs keys [0, wave_key_end)

  // ---- the first global reads, all in flight together: the page ids of the first two address windows (what the K/V
  // loads need first), then this wave's Q rows.  The K/V loads are issued as soon as the page ids are there; Q is
  // staged while they travel.
  // A window is fetched in two parts, so that the page-table read can be in flight while other work goes on: the
  // page id first, the addresses from it later.
  auto window_page = [&](int w) __attribute__((always_inline)) {
    const int gi = w * 64 + lane;
    int page = -1;
    if (gi * SKV_BLOCK_TOKENS < L && gi < p.max_blocks)
      page = __builtin_nontemporal_load(&p.page_table[(size_t)r * p.max_blocks + gi]);
    return page;
  };
  // (the five base addresses as values: selecting between the fields of the argument block itself makes the
  // compiler select their addresses and load through them, a vector-memory read that everything behind it waits for)
  const uint64_t kpool_a = (uint64_t)p.kpool, vpool_a = (uint64_t)p.vpool, knew_a = (uint64_t)p.knew,
                 vnew_a = (uint64_t)p.vnew, zero_a = (uint64_t)p.zero_page;
  auto window_bases = [&](int w, int page, uint64_t& ak, uint64_t& av) __attribute__((always_inline)) {
    const int gi = w * 64 + lane;
    const int key0 = gi * SKV_BLOCK_TOKENS;
    uint64_t k = zero_a, v = zero_a;
    if (key0 < L) {
      if (page >= 0 && page < p.n_pages) {
        const uint64_t off = ((uint64_t)page * SKV_BLOCK_TOKENS * p.Hkv + kvh) * (kD * 2);
        k = kpool_a + off;
        v = vpool_a + off;
      }
    } else if (key0 < Ltot) {
      const uint64_t off = ((uint64_t)(qbase + key0 - L) * p.Hkv + kvh) * (kD * 2);
      k = knew_a + off;
      v = vnew_a + off;
    }
    ak = k;
    av = v;
  };
  const int page_w0 = window_page(0), page_w1 = window_page(1);

  // ---- Q fragments (B operand of S^T = K Q^T): lane holds query l32, d = 16 ks + 8 half .. +7
  // Rows are fetched whole (16 lanes x 16 B per row) and picked up from the wave's staging tile.  The scores leave the
  // matrix core unscaled; scale * log2(e) is applied in fp32 by the multiply-add that also subtracts the reference
  // (scaling Q itself would round it to bf16 a second time: visible when scores spread over hundreds of units).
  const float c = p.scale * kLog2e;
  bf16x8 qf[8];
  u32x4 qv[8];
  {
    const int c16 = lane & 15;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rr = (lane >> 4) + 4 * i;
      const int row = min(pos0 + rr, S - 1);   // rows past the tile or the request are computed and dropped
      qv[i] = *(const u32x4*)((const __bf16*)p.q + ((size_t)(qbase + row) * p.Hq + head) * kD + c16 * 8);
    }
  }
  auto stage_q = [&]() __attribute__((always_inline)) {
    const int c16 = lane & 15;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {   // the staging tile takes 16 rows at a time
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rr = (lane >> 4) + 4 * i;    // row within the pass
        *(u32x4*)(stage + rr * kD + ((c16 ^ rr) << 3)) = qv[4 * pass + i];
      }
      if ((l32 >> 4) == pass) {
        const int rr = l32 & 15;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const bf16x8*)(stage + rr * kD + (((2 * ks + half) ^ rr) << 3));
      }
    }
  };

  f32x16 o[4];   // O^T accumulators: d = 32 a + 8(e/4) + 4 half + e%4, query = l32
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[a][e] = 0.f;

  // ---- global -> LDS, without a stop in registers ----
  // A tile is four 16-key groups; a group is one page of the pool or 16 consecutive new rows.  Each wavefront
  // moves two segments of a tile (segments w and w + 8: keys 4w.. and 32 + 4w..) with direct-to-LDS loads: lane i
  // fetches chunk 4 (i / 16) + i % 4 of key (i / 4) % 4 of the segment and the hardware puts it at slot i.
  const unsigned row_bytes = (unsigned)p.Hkv * kD * 2u;
  const int t_row = (wave & 3) * 4 + ((lane >> 2) & 3);      // row of the 16-key group this lane fetches
  const unsigned t_col = (unsigned)((lane >> 4) * 4 + (lane & 3)) * 16u;
  const unsigned t_off = (unsigned)t_row * row_bytes + t_col;
  // Group base addresses, one 16-key group per lane for 64 groups (16 tiles, a "window"): a pool page, 16 new rows,
  // or the page of zeros when the group has no data (past the end of the sequence, or a page id outside the pool).
  // A tile's bases are read with lane broadcasts.  Two consecutive windows are held; K tiles run one tile ahead of
  // V tiles, so for one iteration in sixteen K reads the later window while V still reads the earlier one.
  auto lane_bcast = [&](uint64_t x, int idx) __attribute__((always_inline)) {
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)x, idx);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), idx);
    return (const __attribute__((address_space(1))) char*)(((uint64_t)hi << 32) | lo);   // global, not flat
  };
  uint64_t ak_cur, av_cur, ak_nxt, av_nxt;
  int win = 0;                       // window held in *_cur; *_nxt holds window win + 1
  window_bases(0, page_w0, ak_cur, av_cur);
  window_bases(1, page_w1, ak_nxt, av_nxt);
  typedef __attribute__((address_space(3))) void lds_void;
  // one pool (K or V) of tile t into an LDS stage; `bases` holds the window of tile t
  auto load_half_tile = [&](uint64_t bases, int t, __bf16* dst_stage) __attribute__((always_inline)) {
    const int key_base = t * kBN;
    __bf16* const dst = dst_stage + wave * kSeg;
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const int g = (wave >> 2) + 2 * cc;                    // 16-key group of segment wave + 8 cc
      const int idx = ((t & 15) << 2) + g;
      const auto gb = lane_bcast(bases, idx);
      unsigned off = t_off;
      if (key_base + kBN > Ltot) {  // the sequence ends inside this tile: rows past its end re-read its last row,
        const int n_valid = Ltot - (key_base + g * 16);  // finite values that the causal mask keeps out
        if (n_valid > 0 && n_valid < 16) off = (unsigned)min(t_row, n_valid - 1) * row_bytes + t_col;
      }
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gb + off),
                                       (lds_void*)(dst + cc * 8 * kSeg), 16, 0, 0);
    }
  };
  auto load_k_tile = [&](int t, int stage_idx) __attribute__((always_inline)) {
    load_half_tile((t >> 4) == win ? ak_cur : ak_nxt, t, Ks + stage_idx * kTile);
  };
  auto load_v_tile = [&](int t, int stage_idx) __attribute__((always_inline)) {
    load_half_tile((t >> 4) == win ? av_cur : av_nxt, t, Vs + stage_idx * kTile);
  };
  // Inside the main loop the same loads are split in two: the segment bases of the tiles an iteration will request
  // (K two tiles ahead, V one) are broadcast out of the windows during the iteration before, between its half-steps,
  // so that the iteration itself starts with nothing but the four load instructions.  Right after a barrier every
  // wave of the workgroup is at this point at once, and what stands here keeps all matrix cores waiting.
  typedef const __attribute__((address_space(1))) char* gptr;
  gptr nk[2], nv[2];
  int pend_page = -1;
  bool pend = false;
  auto prep_bases = [&](int kt_next) __attribute__((always_inline)) {
    if (((kt_next + 1) >> 4) != win) {   // V enters the next window: move on and ask for the page ids of the one
      ++win;                             // after it; K needs that window fourteen iterations from now, the iteration
      ak_cur = ak_nxt;                   // after this one turns the ids into addresses, behind its barrier, where
      av_cur = av_nxt;                   // every load of this wave has landed anyway
      pend_page = window_page(win + 1);
      pend = true;
    }
    const int tk = kt_next + 2, tv = kt_next + 1;
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const int g = (wave >> 2) + 2 * cc;
      nk[cc] = lane_bcast((tk >> 4) == win ? ak_cur : ak_nxt, ((tk & 15) << 2) + g);
      nv[cc] = lane_bcast((tv >> 4) == win ? av_cur : av_nxt, ((tv & 15) << 2) + g);
    }
  };
  auto issue_half_tile = [&]<bool kWhole>(const gptr (&b)[2], int t, __bf16* dst_stage) __attribute__((always_inline)) {
    const int key_base = t * kBN;
    __bf16* const dst = dst_stage + wave * kSeg;
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      unsigned off = t_off;
      if (!kWhole && key_base + kBN > Ltot) {   // as in load_half_tile
        const int n_valid = Ltot - (key_base + ((wave >> 2) + 2 * cc) * 16);
        if (n_valid > 0 && n_valid < 16) off = (unsigned)min(t_row, n_valid - 1) * row_bytes + t_col;
      }
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(b[cc] + off),
                                       (lds_void*)(dst + cc * 8 * kSeg), 16, 0, 0);
    }
  };
  // a wave's direct loads are in LDS once its vector-memory counter has drained; the barrier then publishes them
  auto tile_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  // ---- the steps of the pipeline ----
  // Work advances in 32-key sub-tiles (half an LDS tile), three of them in flight: half-step h puts the scores of
  // sub-tile h + 1 and the output update with sub-tile h - 1 on the matrix core and computes the softmax of sub-tile
  // h on the vector ALU.  Nothing inside a half-step depends on anything else inside it, so its 16 MFMAs alternate
  // (score, output, score, ...) with two or three vector instructions behind each: the vector work runs beside the
  // MFMAs instead of between them.  Two score accumulators and two P^T buffers alternate.
  f32x16 s[2];      // S^T of two consecutive sub-tiles: [32 keys][32 queries], raw dot products
  bf16x8 pb[2][2];  // P^T as B operands: [sub-tile parity][16-key group]
  bf16x8 kfr[4];    // K fragment ring: runs four fragments ahead, across sub-tiles
  bf16x8 vfr[4];    // V^T fragment ring, likewise
  float m_ref = 0.f;   // reference the exponentials are taken against (score * scale * log2(e): exp2 units), per query
  float l_run = 0.f;   // running row sum over this lane-half's keys
#pragma unroll
  for (int e = 0; e < 16; ++e) s[0][e] = s[1][e] = 0.f;
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int e = 0; e < 8; ++e) pb[0][0][e] = pb[0][1][e] = pb[1][0][e] = pb[1][1][e] = (__bf16)0.f;
  // K fragment (ks, mt): lane (l32, half) wants key l32 + 32 mt, chunk 2 ks + half.  In bf16 elements:
  //   segment (l32 / 4 + 8 mt) * kSeg + key-in-segment (l32 % 4) * 32 + (ks / 2) * 128 + (2 (ks % 2) + half) * 8
  const int k_lane = (l32 >> 2) * kSeg + (l32 & 3) * 32 + half * 8;
  // The PV A operand wants, per lane (d = 32 a + l32), the eight keys {4 half + 0..3, 8 + 4 half + 0..3}
  // of a 16-key group -- the keys this lane-half's P^T registers hold.  Each quad comes from one LDS
  // transpose load: within 16 lanes, lane i supplies the address of 4 consecutive d of key (i / 4) at d
  // offset 4 (i % 4) and receives d offset i of the four keys.  For fragment (g16, a) the lane's key is
  // 16 g16 + 4 half + (lane % 16) / 4 (segment 4 g16 + half, second load two segments on) and its 8 bytes are piece
  // lane % 2 of chunk 4 a + 2 ((lane / 16) % 2) + (lane % 4) / 2.
  const int v_lane = half * kSeg + ((lane & 15) >> 2) * 32 + (2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) * 8 + 4 * (lane & 1);
  // fragment addresses are LDS byte addresses: a per-lane base plus constants that fit the offset field
  auto k_frag = [&](uint32_t kb, int ks) __attribute__((always_inline)) {   // kb: stage + k_lane + mt * 8 kSeg
    return lds_read_b128(kb, ((ks >> 1) * 128 + (ks & 1) * 16) * 2);
  };
  auto v_frag = [&](uint32_t vb, int j) __attribute__((always_inline)) {   // vb: stage + v_lane + h * 8 kSeg; j = (g, a)
    const int off = ((j >> 2) * 4 * kSeg + (j & 3) * 128) * 2;
    const s16x4 lo = lds_read_tr16_b64(vb, off);
    const s16x4 hi = lds_read_tr16_b64(vb, off + 2 * kSeg * 2);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  // causal mask of sub-tile u (keys 32 u ..), applied where the sub-tile reaches past the wave's first row
  auto mask = [&](f32x16& x, int u) __attribute__((always_inline)) {
    const int key0 = u * 32;
    if (key0 + 31 > L + pos0) {
      const int limit = L + pos0 + l32;  // last visible key of this lane's query
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = key0 + (e >> 2) * 8 + half * 4 + (e & 3);
        if (key > limit) x[e] = -INFINITY;
      }
    }
  };
  auto row_max = [&](const f32x16& x) __attribute__((always_inline)) {
    float m4[4];   // four independent reduction chains
#pragma unroll
    for (int k = 0; k < 4; ++k) m4[k] = fmaxf(x[k], x[k + 4]);
#pragma unroll
    for (int e = 8; e < 16; ++e) m4[e & 3] = fmaxf(m4[e & 3], x[e]);
    float mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
    return max_halves(mx);
  };
  // exponentials of one pair of scores -> packed bf16, plain fp32 adds for the row sum (the packed dot-product
  // instruction that would add the pair in one step does not run beside the MFMAs, the adds do)
  float ssum[2];
  bf16x8 pk;
  auto exp_pair = [&](const f32x16& cur, int i, bf16x8 (&p_make)[2], float& e0, float& e1, int part) __attribute__((always_inline)) {
    if (part == 0) {
      e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[2 * i], c, -m_ref));
      e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[2 * i + 1], c, -m_ref));
    } else {
      f32x2 pr = {e0, e1};
      const bf16x2 cv = __builtin_convertvector(pr, bf16x2);
      ssum[0] += e0;
      ssum[1] += e1;
      pk[2 * (i & 3)] = cv[0];
      pk[2 * (i & 3) + 1] = cv[1];
      if ((i & 3) == 3) p_make[i >> 2] = pk;
    }
  };
  // The softmax keeps a reference per query; exponentials are taken against it as it stands, which leaves the
  // normalised result unchanged.  Only when a lane's sum of exponentials over a sub-tile passes kSumLimit (an element
  // at least kSumLimit / 16 above the reference; infinities and NaNs trip it too) is the reference moved to that
  // sub-tile's row maximum: O and the row sum are rescaled and this sub-tile's exponentials are taken again.  This
  // happens between half-steps, after the output update that still belongs to the old reference has been issued.
  auto move_reference = [&](const f32x16& cur, bf16x8 (&p_make)[2]) __attribute__((always_inline)) {
    const float mx = row_max(cur) * c;
    const bool trip = !(max_halves(ssum[0] + ssum[1]) <= kSumLimit);
    const float m_new = trip ? mx : m_ref;
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
    m_ref = m_new;
    l_run *= alpha;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[a][e] *= alpha;
    ssum[0] = ssum[1] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float e0, e1;
      exp_pair(cur, i, p_make, e0, e1, 0);
      exp_pair(cur, i, p_make, e0, e1, 1);
    }
  };
  auto active = [&](int u) __attribute__((always_inline)) { return u * 32 < wave_key_end; };
  // One half-step.  kb / kb_next: K of sub-tiles h + 1 and h + 2; vb / vb_next: V of sub-tiles h - 1 and h.
  // The rings hold fragments 0..3 of sub-tile h + 1 (K) and of sub-tile h - 1 (V^T) on entry and are refilled behind
  // each MFMA with fragments 4..7 and then with fragments 0..3 of the following sub-tile.
  // Fast form (every stage at work, no masked key in sub-tile h): the 16 MFMAs alternate and carry the softmax between
  // them; a fragment is waited for four pair-steps after its request, with eleven (K) or ten (V^T) younger reads.
  auto half_step_fast = [&]<bool kMask>(int h, uint32_t kb, uint32_t kb_next, uint32_t vb, uint32_t vb_next, f32x16& dst,
                                        f32x16& cur, bf16x8 (&p_use)[2], bf16x8 (&p_make)[2]) __attribute__((always_inline)) {
    if (kMask) mask(cur, h);
    ssum[0] = ssum[1] = 0.f;
    // One exponential behind every MFMA, never two in a row: the transcendental unit takes about four issue slots
    // per instruction but works beside the issue port, so a second one right behind the first would hold the
    // wavefront until the unit is free again.  The pair is packed and summed one step later, behind the next
    // exponential.
    float e0 = 0.f, e1 = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      lds_wait(11, kfr[i & 3]);
      dst = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[i & 3], qf[i], i == 0 ? zero16 : dst, 0, 0, 0);
      kfr[i & 3] = i < 4 ? k_frag(kb, i + 4) : k_frag(kb_next, i - 4);
      const float f0 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[2 * i], c, -m_ref));
      if (i > 0) {
        f32x2 pr = {e0, e1};
        const bf16x2 cv = __builtin_convertvector(pr, bf16x2);
        pk[2 * ((i - 1) & 3)] = cv[0];
        pk[2 * ((i - 1) & 3) + 1] = cv[1];
        ssum[0] += e0;
      }
      __builtin_amdgcn_sched_barrier(0);
      lds_wait(10, vfr[i & 3]);
      o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[i & 3], p_use[i >> 2], o[i & 3], 0, 0, 0);
      vfr[i & 3] = i < 4 ? v_frag(vb, i + 4) : v_frag(vb_next, i - 4);
      const float f1 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[2 * i + 1], c, -m_ref));
      if (i > 0) {
        ssum[1] += e1;
        if (((i - 1) & 3) == 3) p_make[(i - 1) >> 2] = pk;
      }
      e0 = f0;
      e1 = f1;
      __builtin_amdgcn_sched_barrier(0);
    }
    {
      f32x2 pr = {e0, e1};
      const bf16x2 cv = __builtin_convertvector(pr, bf16x2);
      pk[6] = cv[0];
      pk[7] = cv[1];
      ssum[0] += e0;
      ssum[1] += e1;
      p_make[1] = pk;
    }
    if (__builtin_expect(__any(!(ssum[0] + ssum[1] <= kSumLimit)), 0)) move_reference(cur, p_make);
    l_run += ssum[0] + ssum[1];
  };
  // General form (first and last iterations of a wave): each stage is tested, runs as a block of its own, and waits
  // for every outstanding read.
  auto half_step_slow = [&](int h, uint32_t kb, uint32_t kb_next, uint32_t vb, uint32_t vb_next, f32x16& dst,
                            f32x16& cur, bf16x8 (&p_use)[2], bf16x8 (&p_make)[2]) __attribute__((always_inline)) {
    if (active(h + 1)) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        lds_wait(0, kfr[i & 3]);
        dst = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[i & 3], qf[i], i == 0 ? zero16 : dst, 0, 0, 0);
        kfr[i & 3] = i < 4 ? k_frag(kb, i + 4) : k_frag(kb_next, i - 4);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (h > 0 && active(h - 1)) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        lds_wait(0, vfr[i & 3]);
        o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[i & 3], p_use[i >> 2], o[i & 3], 0, 0, 0);
        vfr[i & 3] = i < 4 ? v_frag(vb, i + 4) : v_frag(vb_next, i - 4);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) vfr[j] = v_frag(vb_next, j);   // the ring enters the next half-step as it expects
      __builtin_amdgcn_sched_barrier(0);
    }
    if (active(h)) {
      mask(cur, h);
      ssum[0] = ssum[1] = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float e0, e1;
        exp_pair(cur, i, p_make, e0, e1, 0);
        exp_pair(cur, i, p_make, e0, e1, 1);
      }
      if (__builtin_expect(__any(!(ssum[0] + ssum[1] <= kSumLimit)), 0)) move_reference(cur, p_make);
      l_run += ssum[0] + ssum[1];
    }
    // whatever follows finds every fragment of the rings in place
    lds_wait(0, kfr[0], kfr[1], kfr[2], kfr[3]);
    lds_wait(0, vfr[0], vfr[1], vfr[2], vfr[3]);
  };

  // ---- prologue: tiles K(0), K(1), V(0); scores of sub-tile 0; the reference starts at its row maxima
  load_k_tile(0, 0);
  if (n_tiles > 1) load_k_tile(1, 1);
  load_v_tile(0, 0);
  stage_q();
  tile_barrier();
  const uint32_t k_base = lds_addr(Ks + k_lane), v_base = lds_addr(Vs + v_lane);
  constexpr uint32_t kStageBytes = kTile * 2, kHalfBytes = 8 * kSeg * 2;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    kfr[j] = k_frag(k_base, j);
    vfr[j] = kfr[j];   // defined; the V^T ring fills itself during half-step 0
  }
  if (active(0)) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      lds_wait(0, kfr[ks & 3]);
      s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ks & 3], qf[ks], ks == 0 ? zero16 : s[0], 0, 0, 0);
      kfr[ks & 3] = ks < 4 ? k_frag(k_base, ks + 4) : k_frag(k_base + kHalfBytes, ks - 4);
      __builtin_amdgcn_sched_barrier(0);
    }
    // (idle states for the last MFMA: the compiler's wait-state insertion does not look through the branch inside
    // mask(), and the row maximum behind it would read score registers the matrix core has not written yet)
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" : "+v"(s[0]));
    mask(s[0], 0);
    m_ref = row_max(s[0]) * c;   // finite: key 0 is visible to every query
  }

  // ---- main loop.  Iteration kt (two half-steps) reads K(kt), K(kt + 1), V(kt - 1), V(kt).  It starts behind the
  // barrier that published K(kt + 1) and V(kt) and behind which no wave still reads K(kt - 1) or V(kt - 2): their
  // stages take the direct loads of K(kt + 2) and V(kt + 1), in flight during the whole iteration.  One barrier per
  // tile; one more iteration than tiles, for the output update with the last sub-tile.
  // Iterations [1, kt_fast) of this wave have all three stages at work, no masked key and no ragged tile to load.
  const int kt_fast = min(min((L + pos0 - 63) / 64 + 1, (wave_key_end - 1) / 64), n_tiles - 3);
  // Iterations [kt_fast, kt_mid) still have all three stages at work in both half-steps, but keys may be masked and
  // the tiles they request may be ragged or absent (the last two or three before the diagonal tile): they run the
  // fast form with the mask applied and the general loads.
  const int kt_mid = (wave_key_end - 1) / 64;
  int st0 = 0;   // stage of K(kt) and V(kt); tile t sits in stage t % 3
  auto iteration = [&]<int kForm>(int kt) __attribute__((always_inline)) {   // 0 general, 1 fast, 2 fast with masks
    constexpr bool kFast = kForm == 1;
    const int st1 = st0 == 2 ? 0 : st0 + 1;    // stage of tile kt + 1
    const int st2 = st1 == 2 ? 0 : st1 + 1;    // stage of tiles kt + 2 and kt - 1
    if (__builtin_expect(pend, 0)) {
      window_bases(win + 1, pend_page, ak_nxt, av_nxt);
      pend = false;
    }
    if (kFast || kt + 2 < n_tiles) issue_half_tile.template operator()<kFast>(nk, kt + 2, Ks + st2 * kTile);
    if (kFast || kt + 1 < n_tiles) issue_half_tile.template operator()<kFast>(nv, kt + 1, Vs + st1 * kTile);
    const uint32_t kb0 = k_base + st0 * kStageBytes;   // K(kt)
    const uint32_t kb1 = k_base + st1 * kStageBytes;   // K(kt + 1)
    const uint32_t vbp = v_base + st2 * kStageBytes;   // V(kt - 1)
    const uint32_t vb0 = v_base + st0 * kStageBytes;   // V(kt)
    if (kForm == 1) {
      half_step_fast.template operator()<false>(2 * kt, kb0 + kHalfBytes, kb1, vbp + kHalfBytes, vb0, s[1], s[0], pb[1], pb[0]);
      prep_bases(kt + 1);
      half_step_fast.template operator()<false>(2 * kt + 1, kb1, kb1 + kHalfBytes, vb0, vb0 + kHalfBytes, s[0], s[1], pb[0], pb[1]);
    } else if (kForm == 2) {
      half_step_fast.template operator()<true>(2 * kt, kb0 + kHalfBytes, kb1, vbp + kHalfBytes, vb0, s[1], s[0], pb[1], pb[0]);
      prep_bases(kt + 1);
      half_step_fast.template operator()<true>(2 * kt + 1, kb1, kb1 + kHalfBytes, vb0, vb0 + kHalfBytes, s[0], s[1], pb[0], pb[1]);
    } else {
      half_step_slow(2 * kt, kb0 + kHalfBytes, kb1, vbp + kHalfBytes, vb0, s[1], s[0], pb[1], pb[0]);
      prep_bases(kt + 1);
      half_step_slow(2 * kt + 1, kb1, kb1 + kHalfBytes, vb0, vb0 + kHalfBytes, s[0], s[1], pb[0], pb[1]);
    }
    tile_barrier();
    st0 = st1;
  };
  int kt = 0;
  prep_bases(0);
  iteration.template operator()<0>(kt++);
  for (; kt < kt_fast; ++kt) iteration.template operator()<1>(kt);
  for (; kt < kt_mid; ++kt) iteration.template operator()<2>(kt);
  for (; kt <= n_tiles; ++kt) iteration.template operator()<0>(kt);

  // ---- normalise and store.  A lane holds query l32 with d = 32 a + 8 (e/4) + 4 half + e%4, i.e. sixteen 8-byte
  // pieces of one output row.  They go through the wave's staging tile, 16 rows at a time, and leave as whole
  // 256-byte rows.
  if (pos0 >= row1) return;
  {
    const float lsum = l_run + swap_halves(l_run);
    const float inv = 1.0f / lsum;
    const int c16 = lane & 15;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      if ((l32 >> 4) == pass) {
        const int rr = l32 & 15;
        __bf16* row = stage + rr * kD;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            f32x2 x0 = {o[a][i4 * 4 + 0] * inv, o[a][i4 * 4 + 1] * inv};
            f32x2 x1 = {o[a][i4 * 4 + 2] * inv, o[a][i4 * 4 + 3] * inv};
            bf16x2 y0 = __builtin_convertvector(x0, bf16x2);
            bf16x2 y1 = __builtin_convertvector(x1, bf16x2);
            u32x2 wv = {__builtin_bit_cast(uint32_t, y0), __builtin_bit_cast(uint32_t, y1)};
            const int chunk = a * 4 + i4;   // d = 8 chunk + 4 half .. + 3
            *(u32x2*)(row + (((chunk ^ rr) << 3) + 4 * half)) = wv;
          }
      }
      // same wave wrote and reads: the LDS operations of one wave complete in order
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rr = (lane >> 4) + 4 * i;   // row within the pass
        const int pos = pos0 + 16 * pass + rr;
        const u32x4 v = *(const u32x4*)(stage + rr * kD + ((c16 ^ rr) << 3));
        if (pos < row1) *(u32x4*)((__bf16*)p.out + ((size_t)(qbase + pos) * p.Hq + head) * kD + c16 * 8) = v;
      }
    }
  }
}

// ---- fp32 kernel: one wavefront per (token, head) output row ----------------------------------
template <int D>
__global__ __launch_bounds__(64) void attn_f32_kernel(AttnParams p, int64_t max_rows) {
  __shared__ float red[64 * (D + 1)];
  const int lane = threadIdx.x;
  const int64_t g = blockIdx.x;  // token row * Hq + head
  const int h = (int)(g % p.Hq);
  const int64_t tok = g / p.Hq;
  if (tok >= max_rows || tok >= p.q_off[p.n_req]) return;
  int lo = 0, hi = p.n_req;  // q_off[lo] <= tok < q_off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (p.q_off[mid] <= tok) lo = mid; else hi = mid;
  }
  const int r = lo;
  const int qbase = p.q_off[r];
  const int i = (int)(tok - qbase);
  const int L = p.matched_len[r] > 0 ? p.matched_len[r] & ~(SKV_BLOCK_TOKENS - 1) : 0;   // whole blocks only
  const int n_keys = L + i + 1;
  const int hk = h / (p.Hq / p.Hkv);
  const float* q = (const float*)p.q + ((size_t)tok * p.Hq + h) * D;
  float qv[D];
#pragma unroll
  for (int c = 0; c < D; ++c) qv[c] = q[c];
  float m = -INFINITY, l = 0.f;
  float acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) acc[c] = 0.f;
  for (int j = lane; j < n_keys; j += 64) {
    const float *kr = nullptr, *vr = nullptr;
    if (j < L) {
      const int page = p.page_table[(size_t)r * p.max_blocks + j / SKV_BLOCK_TOKENS];
      if (page >= 0 && page < p.n_pages) {
        const size_t off = (((size_t)page * SKV_BLOCK_TOKENS + j % SKV_BLOCK_TOKENS) * p.Hkv + hk) * D;
        kr = (const float*)p.kpool + off;
        vr = (const float*)p.vpool + off;
      }
    } else {
      const size_t off = ((size_t)(qbase + j - L) * p.Hkv + hk) * D;
      kr = (const float*)p.knew + off;
      vr = (const float*)p.vnew + off;
    }
    float s = 0.f;
    if (kr) {
#pragma unroll
      for (int c = 0; c < D; c += 4) {
        const float4 kk = *(const float4*)(kr + c);
        s += qv[c] * kk.x + qv[c + 1] * kk.y + qv[c + 2] * kk.z + qv[c + 3] * kk.w;
      }
    }
    s *= p.scale;
    const float m_new = fmaxf(m, s);
    const float alpha = expf(m - m_new);
    const float e = expf(s - m_new);
    l = l * alpha + e;
#pragma unroll
    for (int c = 0; c < D; c += 4) {
      float4 vv = {0.f, 0.f, 0.f, 0.f};
      if (vr) vv = *(const float4*)(vr + c);
      acc[c] = acc[c] * alpha + e * vv.x;
      acc[c + 1] = acc[c + 1] * alpha + e * vv.y;
      acc[c + 2] = acc[c + 2] * alpha + e * vv.z;
      acc[c + 3] = acc[c + 3] * alpha + e * vv.w;
    }
    m = m_new;
  }
  // merge the 64 partial softmaxes
  float mw = m;
  for (int o = 32; o >= 1; o >>= 1) mw = fmaxf(mw, __shfl_xor(mw, o));
  const float f = m == -INFINITY ? 0.f : expf(m - mw);
  float lw = l * f;
  for (int o = 32; o >= 1; o >>= 1) lw += __shfl_xor(lw, o);
#pragma unroll
  for (int c = 0; c < D; ++c) red[lane * (D + 1) + c] = acc[c] * f;
  __syncthreads();
  float* out = (float*)p.out + ((size_t)tok * p.Hq + h) * D;
  for (int c = lane; c < D; c += 64) {
    float sum = 0.f;
    for (int t = 0; t < 64; ++t) sum += red[t * (D + 1) + c];
    out[c] = sum / lw;
  }
}

int heads_per_wg_for(int G) { return G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1); }  // divides kWaves

int check_attn(const skv_attn_desc* d) {
  if (!d) return SKV_EINVAL;
  if (d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads) return SKV_EINVAL;
  if (d->dtype == SKV_BF16) return d->head_dim == kD ? SKV_OK : SKV_EINVAL;
  if (d->dtype == SKV_F32) return (d->head_dim == 64 || d->head_dim == 128) ? SKV_OK : SKV_EINVAL;
  return SKV_EINVAL;
}

int64_t max_items_for(const skv_attn_desc* d, int32_t n_req, int64_t total_q_rows) {
  if (d->dtype != SKV_BF16) return 0;
  const int hpw = heads_per_wg_for(d->n_q_heads / d->n_kv_heads);
  const int pos_per_wg = (kWaves / hpw) * kRowsPerWave;
  return total_q_rows / pos_per_wg + 2 * (int64_t)n_req;   // per request: a short first tile and a ragged last one
}

size_t zero_page_bytes(const skv_attn_desc* d) {
  return d->dtype == SKV_BF16 ? skv_align256((size_t)SKV_BLOCK_TOKENS * d->n_kv_heads * kD * 2) : 0;
}

}  // namespace

extern "C" int skv_prefill_attn_workspace_size(const skv_attn_desc* desc, int32_t n_req,
                                               int64_t total_q_rows, size_t* bytes) {
  int rc = check_attn(desc);
  if (rc) return rc;
  if (n_req < 0 || total_q_rows < 0 || !bytes) return SKV_EINVAL;
  *bytes = 256 + zero_page_bytes(desc) + skv_align256((size_t)max_items_for(desc, n_req, total_q_rows) * kItemInts * sizeof(int32_t));
  return SKV_OK;
}

// Host-checkable argument errors common to both entry points.
static int check_attn_buffers(const void* d_q, const void* d_knew, const void* d_vnew, const int32_t* d_q_off,
                              const void* d_kpool, const void* d_vpool, const int32_t* d_matched_len,
                              const int32_t* d_page_table, int32_t max_blocks, const void* d_out) {
  if (!d_q || !d_knew || !d_vnew || !d_q_off || !d_matched_len || !d_out) return SKV_EINVAL;
  if (max_blocks > 0 && (!d_page_table || !d_kpool || !d_vpool)) return SKV_EINVAL;
  if (((uintptr_t)d_q | (uintptr_t)d_knew | (uintptr_t)d_vnew | (uintptr_t)d_kpool | (uintptr_t)d_vpool |
       (uintptr_t)d_out) & 15)
    return SKV_EINVAL;
  return SKV_OK;
}

// Shared by both entry points: enqueues the schedule kernel and the attention kernel on checked arguments.
static int prefill_attn_enqueue(const skv_attn_desc* desc, int32_t n_req, const void* d_q,
                                const void* d_knew, const void* d_vnew, const int32_t* d_q_off,
                                int64_t total_q_rows, const void* d_kpool, const void* d_vpool,
                                int32_t n_pages, const int32_t* d_matched_len,
                                const int32_t* d_page_table, int32_t max_blocks, void* d_out,
                                void* d_workspace, void* stream) {
  hipStream_t st = (hipStream_t)stream;

  AttnParams p;
  p.q = d_q; p.knew = d_knew; p.vnew = d_vnew; p.kpool = d_kpool; p.vpool = d_vpool; p.out = d_out;
  p.q_off = d_q_off; p.matched_len = d_matched_len; p.page_table = d_page_table;
  p.n_items = (const int32_t*)d_workspace;
  p.zero_page = (const char*)d_workspace + 256;
  p.items = (const int32_t*)((char*)d_workspace + 256 + zero_page_bytes(desc));
  p.n_req = n_req; p.max_blocks = max_blocks; p.n_pages = n_pages;
  p.Hq = desc->n_q_heads; p.Hkv = desc->n_kv_heads;
  p.heads_per_wg = heads_per_wg_for(desc->n_q_heads / desc->n_kv_heads);
  p.scale = skv_softmax_scale(desc);

  if (desc->dtype == SKV_F32) {
    const int64_t rows = total_q_rows * desc->n_q_heads;
    if (rows > 0x7fffffff) return SKV_ERANGE;
    if (desc->head_dim == 64)
      attn_f32_kernel<64><<<(int)rows, 64, 0, st>>>(p, total_q_rows);
    else
      attn_f32_kernel<128><<<(int)rows, 64, 0, st>>>(p, total_q_rows);
    SKV_HIP(hipGetLastError());
    return SKV_OK;
  }

  const int64_t max_items = max_items_for(desc, n_req, total_q_rows);
  const int pos_per_wg = (kWaves / p.heads_per_wg) * kRowsPerWave;
  const int n_hg = (desc->n_q_heads / desc->n_kv_heads) / p.heads_per_wg;
  const int64_t grid = max_items * desc->n_kv_heads * n_hg;
  if (grid > 0x7fffffff || max_items > 0x3fffffff) return SKV_ERANGE;
  attn_schedule_kernel<<<1, 1024, 0, st>>>(n_req, d_q_off, d_matched_len, pos_per_wg, (int)max_items,
                                           (int32_t*)d_workspace, (int32_t*)p.items, (uint4*)p.zero_page,
                                           (int)(zero_page_bytes(desc) / 16));
  SKV_HIP(hipGetLastError());
  attn_bf16_kernel<<<(int)grid, kThreads, 0, st>>>(p);
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_prefill_attn(const skv_attn_desc* desc, int32_t n_req, const void* d_q,
                                const void* d_knew, const void* d_vnew, const int32_t* d_q_off,
                                int64_t total_q_rows, const void* d_kpool, const void* d_vpool,
                                int32_t n_pages, const int32_t* d_matched_len,
                                const int32_t* d_page_table, int32_t max_blocks, void* d_out,
                                void* d_workspace, size_t workspace_bytes, void* stream) {
  int rc = check_attn(desc);
  if (rc) return rc;
  if (n_req < 0 || total_q_rows < 0 || n_pages < 0 || max_blocks < 0) return SKV_EINVAL;
  if (n_req == 0 || total_q_rows == 0) return SKV_OK;
  rc = check_attn_buffers(d_q, d_knew, d_vnew, d_q_off, d_kpool, d_vpool, d_matched_len, d_page_table, max_blocks,
                          d_out);
  if (rc) return rc;
  size_t need = 0;
  skv_prefill_attn_workspace_size(desc, n_req, total_q_rows, &need);
  if (!d_workspace || workspace_bytes < need) return SKV_ENOMEM;
  if ((uintptr_t)d_workspace & 15) return SKV_EINVAL;
  return prefill_attn_enqueue(desc, n_req, d_q, d_knew, d_vnew, d_q_off, total_q_rows, d_kpool, d_vpool, n_pages,
                              d_matched_len, d_page_table, max_blocks, d_out, d_workspace, stream);
}

// ---- the same call for callers that cannot allocate ---------------------------------------------
// The work list and the page of zeros live in a file-scope device array instead of a caller workspace.  Every GPU
// the library runs on holds its own copy of the array at its own address, looked up once per device.
static __device__ __align__(256) unsigned char scratch[SKV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, null until looked up

int scratch_of_current_device(void** out) {
  int dev = -1;
  SKV_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SKV_ERANGE;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    // the array's name is only a host-side stand-in; this is its address on the current device
    SKV_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return SKV_EHIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // racing first calls store the same value
  }
  *out = ptr;
  return SKV_OK;
}
}  // namespace

extern "C" int skv_prefill_attn_static(const skv_attn_desc* desc, int32_t n_req, const void* d_q,
                                       const void* d_knew, const void* d_vnew, const int32_t* d_q_off,
                                       int64_t total_q_rows, const void* d_kpool, const void* d_vpool,
                                       int32_t n_pages, const int32_t* d_matched_len,
                                       const int32_t* d_page_table, int32_t max_blocks, void* d_out,
                                       void* stream) {
  int rc = check_attn(desc);
  if (rc) return rc;
  if (n_req < 0 || total_q_rows < 0 || n_pages < 0 || max_blocks < 0) return SKV_EINVAL;
  if (n_req == 0 || total_q_rows == 0) return SKV_OK;
  rc = check_attn_buffers(d_q, d_knew, d_vnew, d_q_off, d_kpool, d_vpool, d_matched_len, d_page_table, max_blocks,
                          d_out);
  if (rc) return rc;
  size_t need = 0;
  skv_prefill_attn_workspace_size(desc, n_req, total_q_rows, &need);
  if (need > (size_t)SKV_STATIC_SCRATCH_BYTES) return SKV_ERANGE;   // batch too large for the built-in scratch
  void* ws = nullptr;
  rc = scratch_of_current_device(&ws);
  if (rc) return rc;
  // the schedule kernel rewrites the item count, the page of zeros and every record it hands out on each call,
  // so nothing of the previous call's contents is read
  return prefill_attn_enqueue(desc, n_req, d_q, d_knew, d_vnew, d_q_off, total_q_rows, d_kpool, d_vpool, n_pages,
                              d_matched_len, d_page_table, max_blocks, d_out, ws, stream);
}

// ---- measurement aid: what the matrix cores sustain on given operand values ----
// The clock the chip holds under matrix load depends on the values flowing through the multipliers, so the rate a
// kernel can reach is a property of its data as well as of its code.  Every wavefront keeps six (A, B) operand
// pairs of the caller's data in registers and issues the attention kernel's MFMA back to back into four
// accumulators: no memory traffic, no other instructions.  One workgroup of eight wavefronts per compute unit; its
// LDS claim keeps a second workgroup off the unit, so every SIMD runs exactly two wavefronts from start to end.
// With side work, every MFMA is accompanied by what the attention kernel's softmax issues per MFMA at the least --
// its A operand read from LDS (16 bytes per lane), one multiply-add, one exponential, one add and half a packed
// conversion -- on values that depend on nothing the matrix core produces: no dependency on a result, no global
// load, no barrier.  What this form sustains bounds any schedule of that instruction mix.
namespace {
constexpr int kRateMaxBlocks = 512, kRateThreads = 512, kRatePairs = 6, kRateLdsBytes = 96 * 1024;
template <bool kSide>
__global__ __launch_bounds__(kRateThreads) void mfma_rate_kernel(const u32x4* __restrict__ ops, float* __restrict__ sink,
                                                                 int iters) {
  __shared__ u32x4 claim[kRateLdsBytes / 16];
  const size_t lane_id = (size_t)blockIdx.x * kRateThreads + threadIdx.x;
  bf16x8 a[kRatePairs], b[kRatePairs];
#pragma unroll
  for (int i = 0; i < kRatePairs; ++i) {
    const u32x4 x = ops[(lane_id * kRatePairs + i) * 2], y = ops[(lane_id * kRatePairs + i) * 2 + 1];
    a[i] = __builtin_bit_cast(bf16x8, x);
    b[i] = __builtin_bit_cast(bf16x8, y);
  }
  f32x16 c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) c[j][e] = 0.f;
  float t = 0.f;
  if (kSide) {
    // the workgroup's own 96 KB of operand data fill the LDS; a wavefront reads A operands from its own 8 KB of it
    constexpr int kVecs = kRateLdsBytes / 16;
    for (int i = threadIdx.x; i < kVecs; i += kRateThreads) claim[i] = ops[(size_t)blockIdx.x * kVecs + i];
    __syncthreads();
    const uint32_t abase = lds_addr(&claim[(threadIdx.x & 63) + (threadIdx.x >> 6) * 512]);
    bf16x8 ar[4] = {a[0], a[1], a[2], a[3]};   // ring: the read behind MFMA j serves MFMA j + 4
    float x[4], e_prev = 0.f, e_pp = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) x[j] = (float)((threadIdx.x * 37 + j * 101) % 1000) * 0.001f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        lds_wait(3, ar[j & 3]);
        c[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ar[j & 3], b[(j / 4 + j) % kRatePairs], c[j & 3], 0, 0, 0);
        ar[j & 3] = lds_read_b128(abase, (j & 7) * 1024);
        x[j & 3] = __builtin_fmaf(-1.9371f, __builtin_fabsf(x[j & 3]), 1.0f);   // bounded, never settles
        const float e = __builtin_amdgcn_exp2f(x[j & 3]);
        t += e_prev;                       // results are consumed one step late, as in the attention kernel: nothing
        if (j & 1) {                       // waits for the transcendental unit
          f32x2 pr = {e_pp, e_prev};
          const bf16x2 cv = __builtin_convertvector(pr, bf16x2);
          asm volatile("" ::"v"(cv));
        }
        e_pp = e_prev;
        e_prev = e;
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    lds_wait(0, ar[0], ar[1], ar[2], ar[3]);
  } else {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 16; ++j)
        c[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j % kRatePairs], b[(j / 4 + j) % kRatePairs], c[j & 3], 0, 0, 0);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) t += c[j][e];
  volatile uint32_t* used = (volatile uint32_t*)claim;   // the array has to be used to be allocated
  used[threadIdx.x] = __float_as_uint(t);
  sink[lane_id] = __uint_as_float(used[threadIdx.x]);
}
}  // namespace

extern "C" int skv_mfma_rate(const void* d_operands, size_t operand_bytes, int32_t iters, int32_t side_work,
                             float* d_sink, size_t sink_bytes, double* flops, void* stream) {
  if (!d_operands || !d_sink || iters < 1 || ((uintptr_t)d_operands & 15)) return SKV_EINVAL;
  if (side_work != 0 && side_work != 1) return SKV_EINVAL;
  if (operand_bytes < SKV_MFMA_RATE_OPERAND_BYTES || sink_bytes < SKV_MFMA_RATE_SINK_BYTES) return SKV_ENOMEM;
  int dev = 0, cus = 0;
  SKV_HIP(hipGetDevice(&dev));
  SKV_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const int blocks = cus < kRateMaxBlocks ? cus : kRateMaxBlocks;
  if (side_work)
    mfma_rate_kernel<true><<<blocks, kRateThreads, 0, (hipStream_t)stream>>>((const u32x4*)d_operands, d_sink, iters);
  else
    mfma_rate_kernel<false><<<blocks, kRateThreads, 0, (hipStream_t)stream>>>((const u32x4*)d_operands, d_sink, iters);
  SKV_HIP(hipGetLastError());
  if (flops) *flops = (double)blocks * (kRateThreads / 64) * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
  return SKV_OK;
}
