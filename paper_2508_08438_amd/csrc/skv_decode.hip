// Decode-step attention over the paged KV cache: one query token per request attends to every cached token.
//
// SafeKV Section 2.1 (the decode phase reads the cached K/V of all earlier tokens at every step; KV reuse
// changes where those pages come from, not what is computed).  The kernel reads the same pools through the
// same page table as the prefill kernel.  A step moves every cached K and V byte once and does 4*d flops per
// byte pair, so it is HBM bound; the work of one (request, kv head) is split over several workgroups along
// the keys, and a second kernel merges the partial softmax states.
//
// Layout of the products (MFMA 16x16): S^T = K Q^T with the G query heads of the kv head as the 16 columns,
// so one wavefront scores 16 keys for all heads with four v_mfma_f32_16x16x32_bf16; the accumulator registers
// (lane = head, registers = 4 keys) are, after exponentiation, the B operand of O^T += V^T P^T
// (v_mfma_f32_16x16x16_bf16), whose A operand comes from the LDS transpose load.
#include "skv_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kD = 128;
constexpr int kBN = 64;               // keys per LDS tile: 16 per wavefront
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kStages = 2;
constexpr int kKsStride = kD + 8;     // bf16 elements per K row in LDS (conflict-free b128 reads)
constexpr int kVsStride = kD + 32;    // bf16 elements per V row in LDS (conflict-free transpose loads)
constexpr int kMaxG = 16;             // query heads per kv head (the columns of one MFMA tile)
constexpr float kLog2e = 1.4426950408889634f;

struct DecParams {
  const void *q, *kpool, *vpool;
  void* out;
  const int32_t *ctx_len, *page_table;
  const char* zero_page;   // 16 rows of zeros: a page id outside the pool reads as zeros
  float *part_m, *part_l, *part_o;  // [R][Hkv][n_splits][G] (x d for part_o)
  int n_req, max_blocks, n_pages, Hq, Hkv, G, n_splits, tiles_per_split;
  float scale;
};

__global__ __launch_bounds__(kThreads, 2) void decode_attn_kernel(DecParams p) {
  __shared__ __attribute__((aligned(16))) __bf16 smem[kStages * kBN * (kKsStride + kVsStride)];
  __bf16* const Ks = smem;                                // [kStages][kBN][kKsStride]
  __bf16* const Vs = smem + kStages * kBN * kKsStride;    // [kStages][kBN][kVsStride]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15;   // column of the MFMA tiles: the query head
  const int g4 = lane >> 4;    // lane group: keys 4 g4 .. 4 g4 + 3 of the wavefront's 16
  // kv head fastest: the workgroups that read the same pages (each its own 256-byte slice of every token row)
  // are dispatched together, one per XCD, and walk the pages at the same time
  const int kvh = blockIdx.x % p.Hkv;
  const int split = (blockIdx.x / p.Hkv) % p.n_splits;
  const int r = blockIdx.x / (p.n_splits * p.Hkv);
  const int G = p.G;
  int ctx = __builtin_amdgcn_readfirstlane(p.ctx_len[r]);
  ctx = max(0, min(ctx, p.max_blocks * SKV_BLOCK_TOKENS));
  const int t0 = split * p.tiles_per_split;
  const int t1 = min(t0 + p.tiles_per_split, (ctx + kBN - 1) / kBN);
  const float c = p.scale * kLog2e;
  const size_t part = ((size_t)(r * p.Hkv + kvh) * p.n_splits + split) * G;

  if (t0 >= t1) {  // nothing cached in this key range (whole workgroup): an empty partial state
    if (tid < G) {
      if (p.n_splits > 1) {
        p.part_m[part + tid] = -INFINITY;
        p.part_l[part + tid] = 0.f;
      } else {
        __bf16* dst = (__bf16*)p.out + ((size_t)r * p.Hq + kvh * G + tid) * kD;
        for (int d = 0; d < kD; ++d) dst[d] = (__bf16)0.f;
      }
    }
    return;
  }

  // ---- Q fragments (B operand of S^T = K Q^T): lane holds head l16, d = 32 ks + 8 g4 .. +7
  bf16x8 qf[4];
  {
    const __bf16* src = (const __bf16*)p.q + ((size_t)r * p.Hq + kvh * G + min(l16, G - 1)) * kD + 8 * g4;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      qf[ks] = *(const bf16x8*)(src + ks * 32);
      if (l16 >= G)
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[ks][e] = (__bf16)0.f;
    }
  }

  // ---- key-group addresses: lane g of window w holds where keys 16 (4 (t0 + 16 w) + g) .. + 15 start
  const unsigned row_bytes = (unsigned)p.Hkv * kD * 2u;
  auto fetch_window = [&](int w, uint64_t& ak, uint64_t& av) __attribute__((always_inline)) {
    const int gi = (t0 + 16 * w) * 4 + lane;
    uint64_t k = (uint64_t)p.zero_page, v = k;
    if (gi * SKV_BLOCK_TOKENS < ctx && gi < p.max_blocks) {
      const int page = p.page_table[(size_t)r * p.max_blocks + gi];
      if (page >= 0 && page < p.n_pages) {
        const uint64_t off = ((uint64_t)page * SKV_BLOCK_TOKENS * p.Hkv + kvh) * (kD * 2);
        k = (uint64_t)p.kpool + off;
        v = (uint64_t)p.vpool + off;
      }
    }
    ak = k;
    av = v;
  };
  auto lane_bcast = [&](uint64_t x, int idx) __attribute__((always_inline)) {
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)x, idx);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), idx);
    return (void*)(((uint64_t)hi << 32) | lo);
  };
  uint64_t ak_cur, av_cur, ak_nxt = 0, av_nxt = 0;
  fetch_window(0, ak_cur, av_cur);

  // ---- global -> registers -> LDS: 16 threads x 16 B per key row, four 16-key groups per tile.  Buffer
  // loads check each lane's offset against the bytes that exist from the group's base on, so the rows of
  // the last page past ctx come back as zeros, whatever the pool holds there.
  u32x4 kregA[4], vregA[4], kregB[4], vregB[4];  // two tiles in flight: kt+1 (landed or landing) and kt+2
  const int t_row = tid >> 4;
  const unsigned t_off = (unsigned)t_row * row_bytes + (unsigned)(tid & 15) * 16u;
  auto load_tile = [&](int kt, u32x4 (&kreg)[4], u32x4 (&vreg)[4], uint64_t ak_w, uint64_t av_w) __attribute__((always_inline)) {
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      const int idx = (((kt - t0) & 15) << 2) + cc;
      int n_valid = ctx - (kt * kBN + cc * 16);  // clamped to 0..16 on the scalar unit
      asm("s_max_i32 %0, %1, 0\n\ts_min_i32 %0, %0, 16" : "=s"(n_valid) : "s"(n_valid) : "scc");
      const int nrec = n_valid * (int)row_bytes;
      const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(lane_bcast(ak_w, idx), 0, nrec, 0x00020000);
      const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(lane_bcast(av_w, idx), 0, nrec, 0x00020000);
      // cache policy 2 = non-temporal: every byte is used once, so the stream should not displace what L2 holds
      kreg[cc] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rk, (int)t_off, 0, 2));
      vreg[cc] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rv, (int)t_off, 0, 2));
    }
  };
  const int k_lds = t_row * kKsStride + (tid & 15) * 8;
  const int v_lds = t_row * kVsStride + (tid & 15) * 8;
  auto store_tile = [&](int kt, const u32x4 (&kreg)[4], const u32x4 (&vreg)[4]) __attribute__((always_inline)) {
    __bf16* kd = Ks + ((kt - t0) % kStages) * (kBN * kKsStride) + k_lds;
    __bf16* vd = Vs + ((kt - t0) % kStages) * (kBN * kVsStride) + v_lds;
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      *(u32x4*)(kd + cc * 16 * kKsStride) = kreg[cc];
      *(u32x4*)(vd + cc * 16 * kVsStride) = vreg[cc];
    }
  };

  // ---- per-wavefront softmax state over its share of the keys
  f32x4 o[8];  // O^T tiles: d = 16 a + 4 g4 + i, head = l16
#pragma unroll
  for (int a = 0; a < 8; ++a) o[a] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY;  // running maximum of head l16 (raw score units), same in the four lane groups
  float l_run = 0.f;        // running sum over this lane group's keys

  const int k_lane = (16 * wave + l16) * kKsStride + 8 * g4;
  const int v_lane = (16 * wave + 4 * g4 + (l16 >> 2)) * kVsStride + 4 * (l16 & 3);
  auto compute = [&](int kt) __attribute__((always_inline)) {
    const __bf16* kb = Ks + ((kt - t0) % kStages) * (kBN * kKsStride) + k_lane;
    const __bf16* vb = Vs + ((kt - t0) % kStages) * (kBN * kVsStride) + v_lane;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const bf16x8*)(kb + ks * 32), qf[ks], s, 0, 0, 0);
    // The scores are read by vector instructions right behind a branch (the ragged-tile test below).  The compiler's
    // wait-state insertion does not look through that branch, and without the states an MFMA result needs before a
    // vector instruction may read it the row maxima are taken from registers the matrix core has not written yet
    // (seen as run-to-run differences in the last bits).  Twelve idle states cover the four-pass MFMA.
    asm volatile("s_nop 7\n\ts_nop 3" : "+v"(s));
    const int key0 = kt * kBN + 16 * wave + 4 * g4;
    if (kt * kBN + kBN > ctx) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (key0 + i >= ctx) s[i] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    float alpha = 1.f;
    f32x4 pr = {0.f, 0.f, 0.f, 0.f};
    if (m_new != -INFINITY) {
      alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      const float mc = m_new * c;
#pragma unroll
      for (int i = 0; i < 4; ++i) pr[i] = __builtin_amdgcn_exp2f(s[i] * c - mc);
    }
    m_run = m_new;
    l_run = l_run * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
    const bf16x2 p01 = __builtin_convertvector(f32x2{pr[0], pr[1]}, bf16x2);
    const bf16x2 p23 = __builtin_convertvector(f32x2{pr[2], pr[3]}, bf16x2);
    const u32x2 pw = {__builtin_bit_cast(uint32_t, p01), __builtin_bit_cast(uint32_t, p23)};
    const s16x4 pf = __builtin_bit_cast(s16x4, pw);
#pragma unroll
    for (int a = 0; a < 8; ++a) {
      const s16x4 vf = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vb + 16 * a));
      o[a] = o[a] * alpha;
      o[a] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf, pf, o[a], 0, 0, 0);
    }
  };

  // ---- main loop: while tile kt is computed, tile kt+1 sits in one register set (on its way to LDS) and the
  // loads of tile kt+2 are in flight into the other; one barrier per tile.  Window w covers tiles
  // t0 + 16 w .. + 15; the window of tile kt+2 is fetched one iteration before that tile is requested.
  int cur_w = 0;
  auto window_of = [&](int kt, uint64_t& ak, uint64_t& av) __attribute__((always_inline)) {
    const bool nxt = ((kt - t0) >> 4) != cur_w;
    ak = nxt ? ak_nxt : ak_cur;
    av = nxt ? av_nxt : av_cur;
  };
  uint64_t akw, avw;
  load_tile(t0, kregA, vregA, ak_cur, av_cur);
  if (t0 + 1 < t1) load_tile(t0 + 1, kregB, vregB, ak_cur, av_cur);   // tile t0+1 is in window 0 (16 tiles per window)
  store_tile(t0, kregA, vregA);
  __syncthreads();
  auto step = [&](int kt, u32x4 (&k_next)[4], u32x4 (&v_next)[4], u32x4 (&k_far)[4], u32x4 (&v_far)[4]) __attribute__((always_inline)) {
    // k_next holds tile kt+1 (requested one step ago); k_far is free and takes tile kt+2
    if (((kt - t0) >> 4) != cur_w) { cur_w = (kt - t0) >> 4; ak_cur = ak_nxt; av_cur = av_nxt; }
    if (((kt - t0 + 3) & 15) == 0 && kt + 3 < t1) fetch_window((kt - t0 + 3) >> 4, ak_nxt, av_nxt);
    if (kt + 2 < t1) {
      window_of(kt + 2, akw, avw);
      load_tile(kt + 2, k_far, v_far, akw, avw);
    }
    compute(kt);
    if (kt + 1 < t1) store_tile(kt + 1, k_next, v_next);
    __syncthreads();
  };
  for (int kt = t0; kt < t1; kt += 2) {
    step(kt, kregB, vregB, kregA, vregA);
    if (kt + 1 < t1) step(kt + 1, kregA, vregA, kregB, vregB);
  }

  // ---- merge the four wavefronts' states through LDS (the tiles are no longer needed after the last barrier)
  float* red_o = (float*)smem;                       // [kWaves][16][kD]
  float* red_m = red_o + kWaves * kMaxG * kD;        // [kWaves][16]
  float* red_l = red_m + kWaves * kMaxG;
  {
    float lt = l_run + __shfl_xor(l_run, 16);
    lt += __shfl_xor(lt, 32);
    float* dst = red_o + (size_t)(wave * kMaxG + l16) * kD + 4 * g4;
#pragma unroll
    for (int a = 0; a < 8; ++a) *(f32x4*)(dst + 16 * a) = o[a];
    if (g4 == 0) {
      red_m[wave * kMaxG + l16] = m_run;
      red_l[wave * kMaxG + l16] = lt;
    }
  }
  __syncthreads();
  {
    const int head = tid >> 4, d0 = (tid & 15) * 8;
    if (head < G) {
      float ms = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) ms = fmaxf(ms, red_m[w * kMaxG + head]);
      float L = 0.f, acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float mw = red_m[w * kMaxG + head];
        if (mw == -INFINITY) continue;
        const float wgt = __builtin_amdgcn_exp2f((mw - ms) * c);
        L += wgt * red_l[w * kMaxG + head];
        const float* src = red_o + (size_t)(w * kMaxG + head) * kD + d0;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += wgt * src[j];
      }
      if (p.n_splits > 1) {
        if ((tid & 15) == 0) {
          p.part_m[part + head] = ms;
          p.part_l[part + head] = L;
        }
        float* dst = p.part_o + (part + head) * kD + d0;
#pragma unroll
        for (int j = 0; j < 8; ++j) dst[j] = acc[j];
      } else {
        const float inv = L > 0.f ? 1.f / L : 0.f;
        __bf16* dst = (__bf16*)p.out + ((size_t)r * p.Hq + kvh * G + head) * kD + d0;
#pragma unroll
        for (int j = 0; j < 8; ++j) dst[j] = (__bf16)(acc[j] * inv);
      }
    }
  }
}

// Merge of the key splits: one workgroup per (request, query head), one thread per d.
__global__ __launch_bounds__(kD) void decode_merge_kernel(DecParams p) {
  const int r = blockIdx.x / p.Hq, h = blockIdx.x % p.Hq;
  const int kvh = h / p.G, head = h % p.G;
  const int d = threadIdx.x;
  const float c = p.scale * kLog2e;
  const size_t base = (size_t)(r * p.Hkv + kvh) * p.n_splits;
  float ms = -INFINITY;
  for (int s = 0; s < p.n_splits; ++s) ms = fmaxf(ms, p.part_m[(base + s) * p.G + head]);
  float L = 0.f, acc = 0.f;
  for (int s = 0; s < p.n_splits; ++s) {
    const size_t i = (base + s) * p.G + head;
    const float m = p.part_m[i];
    if (m == -INFINITY) continue;  // empty split: its O was never written
    const float wgt = __builtin_amdgcn_exp2f((m - ms) * c);
    L += wgt * p.part_l[i];
    acc += wgt * p.part_o[i * kD + d];
  }
  ((__bf16*)p.out)[((size_t)r * p.Hq + h) * kD + d] = (__bf16)(L > 0.f ? acc / L : 0.f);
}

__global__ void zero_fill_kernel(uint4* p, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

int check_decode(const skv_attn_desc* d) {
  if (!d) return SKV_EINVAL;
  if (d->dtype != SKV_BF16 || d->head_dim != kD) return SKV_EINVAL;
  if (d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads) return SKV_EINVAL;
  if (d->n_q_heads / d->n_kv_heads > kMaxG) return SKV_EINVAL;
  return SKV_OK;
}

// Key splits: about 4096 workgroups, i.e. eight rounds over the 512 workgroup slots of the chip (finer splits
// shorten the tail when contexts differ in length; coarser ones amortise the start-up of a workgroup).
void split_plan(const skv_attn_desc* d, int32_t n_req, int32_t max_blocks, int* n_splits, int* tiles_per_split) {
  const int64_t max_tiles = ((int64_t)max_blocks * SKV_BLOCK_TOKENS + kBN - 1) / kBN;
  const int64_t units = (int64_t)n_req * d->n_kv_heads;
  int64_t want = units > 0 ? (4096 + units - 1) / units : 1;
  if (want > max_tiles) want = max_tiles;
  if (want < 1) want = 1;
  const int64_t tps = max_tiles > 0 ? (max_tiles + want - 1) / want : 1;
  *tiles_per_split = (int)(tps < 1 ? 1 : tps);
  *n_splits = (int)(max_tiles > 0 ? (max_tiles + *tiles_per_split - 1) / *tiles_per_split : 1);
}

size_t zero_bytes(const skv_attn_desc* d) { return skv_align256((size_t)SKV_BLOCK_TOKENS * d->n_kv_heads * kD * 2); }

}  // namespace

extern "C" int skv_decode_attn_workspace_size(const skv_attn_desc* desc, int32_t n_req, int32_t max_blocks,
                                              size_t* bytes) {
  int rc = check_decode(desc);
  if (rc) return rc;
  if (n_req < 0 || max_blocks < 0 || !bytes) return SKV_EINVAL;
  int ns, tps;
  split_plan(desc, n_req, max_blocks, &ns, &tps);
  const size_t G = (size_t)(desc->n_q_heads / desc->n_kv_heads);
  const size_t states = (size_t)n_req * desc->n_kv_heads * ns * G;
  *bytes = zero_bytes(desc) + 2 * skv_align256(states * sizeof(float)) + skv_align256(states * kD * sizeof(float));
  return SKV_OK;
}

extern "C" int skv_decode_attn(const skv_attn_desc* desc, int32_t n_req, const void* d_q, const void* d_kpool,
                               const void* d_vpool, int32_t n_pages, const int32_t* d_ctx_len,
                               const int32_t* d_page_table, int32_t max_blocks, void* d_out, void* d_workspace,
                               size_t workspace_bytes, void* stream) {
  int rc = check_decode(desc);
  if (rc) return rc;
  if (n_req < 0 || n_pages < 0 || max_blocks < 0) return SKV_EINVAL;
  if (n_req == 0) return SKV_OK;
  if (!d_q || !d_ctx_len || !d_out) return SKV_EINVAL;
  if (max_blocks > 0 && (!d_page_table || !d_kpool || !d_vpool)) return SKV_EINVAL;
  if (((uintptr_t)d_q | (uintptr_t)d_kpool | (uintptr_t)d_vpool | (uintptr_t)d_out | (uintptr_t)d_workspace) & 15)
    return SKV_EINVAL;
  size_t need = 0;
  skv_decode_attn_workspace_size(desc, n_req, max_blocks, &need);
  if (!d_workspace || workspace_bytes < need) return SKV_ENOMEM;
  int ns, tps;
  split_plan(desc, n_req, max_blocks, &ns, &tps);
  const int64_t grid = (int64_t)n_req * desc->n_kv_heads * ns;
  if (grid > 0x7fffffff || (int64_t)n_req * desc->n_q_heads > 0x7fffffff) return SKV_ERANGE;
  hipStream_t st = (hipStream_t)stream;
  const size_t G = (size_t)(desc->n_q_heads / desc->n_kv_heads);
  const size_t states = (size_t)n_req * desc->n_kv_heads * ns * G;
  char* ws = (char*)d_workspace;
  DecParams p;
  p.q = d_q; p.kpool = d_kpool; p.vpool = d_vpool; p.out = d_out;
  p.ctx_len = d_ctx_len; p.page_table = d_page_table;
  p.zero_page = ws;
  p.part_m = (float*)(ws + zero_bytes(desc));
  p.part_l = (float*)((char*)p.part_m + skv_align256(states * sizeof(float)));
  p.part_o = (float*)((char*)p.part_l + skv_align256(states * sizeof(float)));
  p.n_req = n_req; p.max_blocks = max_blocks; p.n_pages = n_pages;
  p.Hq = desc->n_q_heads; p.Hkv = desc->n_kv_heads; p.G = (int)G;
  p.n_splits = ns; p.tiles_per_split = tps; p.scale = skv_softmax_scale(desc);
  zero_fill_kernel<<<8, 256, 0, st>>>((uint4*)ws, (int)(zero_bytes(desc) / 16));
  decode_attn_kernel<<<(int)grid, kThreads, 0, st>>>(p);
  SKV_HIP(hipGetLastError());
  if (ns > 1) {
    decode_merge_kernel<<<n_req * desc->n_q_heads, kD, 0, st>>>(p);
    SKV_HIP(hipGetLastError());
  }
  return SKV_OK;
}
