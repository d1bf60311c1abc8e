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
// direct-to-LDS loads (no stop in registers, no LDS store instructions).  The products are
// formed transposed (S^T = K Q^T, O^T = V^T P^T) so that a query is a lane-column of the MFMA
// accumulator: row max / row sum are register reductions plus one cross-half exchange, and
// the P^T accumulator registers are already in the B-operand layout of the second product;
// V^T fragments come from the LDS transpose load.
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
constexpr int kKStages = 2;      // LDS stages of K
constexpr int kVStages = 2;      // LDS stages of V
constexpr float kRescaleLog2 = 8.f;  // move the softmax reference when a row maximum exceeds it by 2^8
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
// no workgroup streams a key tile for the sake of a few keys of round-up.
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

struct Softmax {
  float m_ref;   // reference maximum the exponentials are taken against (raw score units)
  float l_run;   // running row sum over this lane-half's keys
};

__global__ __launch_bounds__(kThreads, 2) void attn_bf16_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) __bf16 smem[kKStages * kTile + kVStages * kTile +
                                                      kWaves * kRowsPerWave * kD];
  __bf16* const Ks = smem;
  __bf16* const Vs = smem + kKStages * kTile;
  // [kWaves][32 rows][16 chunks of 8 bf16]: each wave's own staging tile for its Q rows on the way in and its O rows
  // on the way out, 16-byte chunks XOR-swizzled by row so that row-wise and fragment-wise accesses are conflict free
  __bf16* const stage = Vs + kVStages * kTile + (threadIdx.x >> 6) * (kRowsPerWave * kD);

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

  // ---- Q fragments (B operand of S^T = K Q^T): lane holds query l32, d = 16 ks + 8 half .. +7
  // Rows are fetched whole (16 lanes x 16 B per row) into the wave's staging tile and picked up from there.
  bf16x8 qf[8];
  {
    const int c16 = lane & 15;
    u32x4 qv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rr = (lane >> 4) + 4 * i;
      const int row = min(pos0 + rr, S - 1);   // rows past the tile or the request are computed and dropped
      qv[i] = *(const u32x4*)((const __bf16*)p.q + ((size_t)(qbase + row) * p.Hq + head) * kD + c16 * 8);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rr = (lane >> 4) + 4 * i;
      *(u32x4*)(stage + rr * kD + ((c16 ^ (rr & 15)) << 3)) = qv[i];
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const bf16x8*)(stage + l32 * kD + (((2 * ks + half) ^ (l32 & 15)) << 3));
  }

  f32x16 o[4];   // O^T accumulators: d = 32 a + 8(e/4) + 4 half + e%4, query = l32
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[a][e] = 0.f;
  Softmax sm{-INFINITY, 0.f};
  const float c = p.scale * kLog2e;
  const float thr = kRescaleLog2 / c;  // raw-score distance above the reference that forces a rescale

  // ---- global -> LDS, without a stop in registers ----
  // A tile is four 16-key groups; a group is one page of the pool or 16 consecutive new rows.  Each wavefront
  // moves two K and two V segments of a tile (segments w and w + 8: keys 4w.. and 32 + 4w..) with direct-to-LDS
  // loads: lane i fetches chunk 4 (i / 16) + i % 4 of key (i / 4) % 4 of the segment and the hardware puts it at slot i.
  const unsigned row_bytes = (unsigned)p.Hkv * kD * 2u;
  const int t_row = (wave & 3) * 4 + ((lane >> 2) & 3);      // row of the 16-key group this lane fetches
  const unsigned t_col = (unsigned)((lane >> 4) * 4 + (lane & 3)) * 16u;
  const unsigned t_off = (unsigned)t_row * row_bytes + t_col;
  // Group base addresses, one 16-key group per lane for the next 64 groups (16 tiles): a pool page, 16 new rows,
  // or the page of zeros when the group has no data (past the end of the sequence, or a page id outside the pool).
  // A tile's bases are read with lane broadcasts.  Window w is fetched one iteration before its first use.
  auto fetch_window = [&](int w, uint64_t& ak, uint64_t& av) __attribute__((always_inline)) {
    const int gi = w * 64 + lane;
    const int key0 = gi * SKV_BLOCK_TOKENS;
    uint64_t k = (uint64_t)p.zero_page, v = k;
    if (key0 < L) {
      if (gi < p.max_blocks) {
        const int page = p.page_table[(size_t)r * p.max_blocks + gi];
        if (page >= 0 && page < p.n_pages) {
          const uint64_t off = ((uint64_t)page * SKV_BLOCK_TOKENS * p.Hkv + kvh) * (kD * 2);
          k = (uint64_t)p.kpool + off;
          v = (uint64_t)p.vpool + off;
        }
      }
    } else if (key0 < Ltot) {
      const uint64_t off = ((uint64_t)(qbase + key0 - L) * p.Hkv + kvh) * (kD * 2);
      k = (uint64_t)p.knew + off;
      v = (uint64_t)p.vnew + off;
    }
    ak = k;
    av = v;
  };
  auto lane_bcast = [&](uint64_t x, int idx) __attribute__((always_inline)) {
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)x, idx);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), idx);
    return (const __attribute__((address_space(1))) char*)(((uint64_t)hi << 32) | lo);   // global, not flat
  };
  uint64_t ak_cur, av_cur, ak_nxt = 0, av_nxt = 0;
  fetch_window(0, ak_cur, av_cur);
  typedef __attribute__((address_space(3))) void lds_void;
  auto load_tile = [&](int kt) __attribute__((always_inline)) {
    const int key_base = kt * kBN;
    __bf16* const kdst = Ks + (kt % kKStages) * kTile + wave * kSeg;
    __bf16* const vdst = Vs + (kt % kVStages) * kTile + wave * kSeg;
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const int g = (wave >> 2) + 2 * cc;                    // 16-key group of segment wave + 8 cc
      const int idx = ((kt & 15) << 2) + g;
      const auto kb = lane_bcast(ak_cur, idx);
      const auto vb = lane_bcast(av_cur, idx);
      unsigned off = t_off;
      if (key_base + kBN > Ltot) {  // the sequence ends inside this tile: rows past its end re-read its last row,
        const int n_valid = Ltot - (key_base + g * 16);  // finite values that the causal mask keeps out
        if (n_valid > 0 && n_valid < 16) off = (unsigned)min(t_row, n_valid - 1) * row_bytes + t_col;
      }
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kb + off),
                                       (lds_void*)(kdst + cc * 8 * kSeg), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vb + off),
                                       (lds_void*)(vdst + cc * 8 * kSeg), 16, 0, 0);
    }
  };
  // a wave's direct loads are in LDS once its vector-memory counter has drained; the barrier then publishes them
  auto tile_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  // ---- the phases of a tile ----
  // LDS fragment reads run eight fragments ahead of the MFMAs that consume them (a fragment register
  // is refilled as soon as its MFMA has been issued), and the first V fragments are requested before
  // the softmax, so that LDS latency hides behind matrix-core and vector work.
  f32x16 s[2];   // S^T of the current tile: [64 keys][32 queries] as two 32x32 tiles
  bf16x8 pb[4];  // P^T as B operands, one per 16-key group
  bf16x8 fr[8];  // fragment ring: K fragments during QK, V^T fragments during PV
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
  auto k_frag = [&](const __bf16* kb, int j) __attribute__((always_inline)) {   // fragment j = (ks, mt) = (j / 2, j % 2)
    return *(const bf16x8*)(kb + (j & 1) * 8 * kSeg + (j >> 2) * 128 + ((j >> 1) & 1) * 16);
  };
  auto v_frag = [&](const __bf16* vb, int j) __attribute__((always_inline)) {   // fragment j = (g16, a) = (j / 4, j % 4)
    const __bf16* src = vb + (j >> 2) * 4 * kSeg + (j & 3) * 128;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src + 2 * kSeg));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  // S^T = K Q^T, then the causal mask on tiles that reach past the first row's limit
  auto qk = [&](int kt) __attribute__((always_inline)) {
    const __bf16* kb = Ks + (kt % kKStages) * kTile + k_lane;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) fr[j] = k_frag(kb, j);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int ks = j >> 1, mt = j & 1;
      s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 7], qf[ks], ks == 0 ? zero : s[mt], 0, 0, 0);
      if (j < 8) fr[j] = k_frag(kb, j + 8);
      __builtin_amdgcn_sched_barrier(0);
    }
    const int key_base = kt * kBN;
    if (key_base + kBN - 1 > L + pos0) {
      const int limit = L + pos0 + l32;  // last visible key of this lane's query
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = key_base + mt * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
          if (key > limit) s[mt][e] = -INFINITY;
        }
    }
  };
  // Streaming softmax: the reference maximum only moves when a row maximum exceeds it by more than
  // 2^kRescaleLog2 (then O and the row sum are rescaled); otherwise exponentials are taken against
  // the stale reference, which leaves the normalised result unchanged.
  auto softmax = [&]() __attribute__((always_inline)) {
    float m4[4];   // four independent reduction chains
#pragma unroll
    for (int k = 0; k < 4; ++k) m4[k] = fmaxf(s[0][k], s[1][k]);
#pragma unroll
    for (int e = 4; e < 16; ++e) m4[e & 3] = fmaxf(m4[e & 3], fmaxf(s[0][e], s[1][e]));
    float mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
    mx = fmaxf(mx, swap_halves(mx));
    if (__any(mx > sm.m_ref + thr)) {
      const float m_new = fmaxf(sm.m_ref, mx);
      const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f((sm.m_ref - m_new) * c);
      sm.m_ref = m_new;
      sm.l_run *= alpha;
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[a][e] *= alpha;
    }
    const float mc = sm.m_ref * c;
    float sum4[4] = {0.f, 0.f, 0.f, 0.f};   // one partial row sum per 16-key group: independent chains
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int q2 = 0; q2 < 2; ++q2) {
        bf16x8 pk;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const float e0 = __builtin_amdgcn_exp2f(s[mt][q2 * 8 + e] * c - mc);
          const float e1 = __builtin_amdgcn_exp2f(s[mt][q2 * 8 + e + 1] * c - mc);
          sum4[mt * 2 + q2] += e0 + e1;
          f32x2 pr = {e0, e1};
          bf16x2 cv = __builtin_convertvector(pr, bf16x2);
          pk[e] = cv[0];
          pk[e + 1] = cv[1];
        }
        pb[mt * 2 + q2] = pk;
      }
    sm.l_run += (sum4[0] + sum4[1]) + (sum4[2] + sum4[3]);
  };
  // O^T += V^T P^T : [128 d][32 queries]
  auto pv_prefetch = [&](int kt) __attribute__((always_inline)) {
    const __bf16* vb = Vs + (kt % kVStages) * kTile + v_lane;
#pragma unroll
    for (int j = 0; j < 8; ++j) fr[j] = v_frag(vb, j);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto pv = [&](int kt) __attribute__((always_inline)) {
    const __bf16* vb = Vs + (kt % kVStages) * kTile + v_lane;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int g16 = j >> 2, a = j & 3;
      o[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j & 7], pb[g16], o[a], 0, 0, 0);
      if (j < 8) fr[j] = v_frag(vb, j + 8);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- main loop: the direct loads of tile kt+1 are in flight during the math on tile kt; one barrier per tile
  load_tile(0);
  tile_barrier();
  for (int kt = 0; kt < n_tiles; ++kt) {
    if (((kt + 1) & 15) == 0) { ak_cur = ak_nxt; av_cur = av_nxt; }
    // the other stage was last read one iteration ago, before the barrier every wave has passed
    if (kt + 1 < n_tiles) load_tile(kt + 1);
    if (((kt + 2) & 15) == 0) fetch_window((kt + 2) >> 4, ak_nxt, av_nxt);
    if (kt * kBN < wave_key_end) {
      qk(kt);
      pv_prefetch(kt);
      softmax();
      pv(kt);
    }
    tile_barrier();
  }

  // ---- normalise and store.  A lane holds query l32 with d = 32 a + 8 (e/4) + 4 half + e%4, i.e. sixteen 8-byte
  // pieces of one output row.  They go through the wave's staging tile and leave as whole 256-byte rows.
  if (pos0 >= row1) return;
  {
    const float lsum = sm.l_run + swap_halves(sm.l_run);
    const float inv = 1.0f / lsum;
    {
      __bf16* row = stage + l32 * kD;
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
          *(u32x2*)(row + (((chunk ^ (l32 & 15)) << 3) + 4 * half)) = wv;
        }
    }
    // same wave wrote and reads: the LDS operations of one wave complete in order
    const int c16 = lane & 15;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int rr = (lane >> 4) + 4 * i;   // row of this wave's tile
      const int pos = pos0 + rr;
      const u32x4 v = *(const u32x4*)(stage + rr * kD + ((c16 ^ (rr & 15)) << 3));
      if (pos < row1) *(u32x4*)((__bf16*)p.out + ((size_t)(qbase + pos) * p.Hq + head) * kD + c16 * 8) = v;
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
