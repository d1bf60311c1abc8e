// Page-table gather of the reused KV pages into per-request contiguous staging.
//
// SafeKV Section 4.3.2: after the lookup stops at a compressed node the required KV blocks are
// read directly from its address vector.  Here the address vector is the page table written by
// the match; a page is one contiguous chunk of 16 * n_kv_heads * head_dim elements, so the
// gather is a batch of page-sized copies chosen by the table.  Workgroups loop over the global
// list of matched pages (persistent grid), each page moving as 16-byte vectors with all loads
// of a step issued before its stores.
#include "skv_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 8;  // 16-byte vectors in flight per thread and pool

__global__ void ctx_offsets_kernel(int n_req, const int32_t* __restrict__ matched_len,
                                   int64_t* __restrict__ ctx_off) {
  __shared__ int64_t sh[1024];
  __shared__ int64_t carry;
  if (threadIdx.x == 0) { carry = 0; ctx_off[0] = 0; }
  __syncthreads();
  for (int base = 0; base < n_req; base += 1024) {
    const int r = base + threadIdx.x;
    int64_t v = 0;
    if (r < n_req) v = matched_len[r] > 0 ? (matched_len[r] / SKV_BLOCK_TOKENS) * SKV_BLOCK_TOKENS : 0;
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      int64_t add = threadIdx.x >= o ? sh[threadIdx.x - o] : 0;
      __syncthreads();
      sh[threadIdx.x] += add;
      __syncthreads();
    }
    if (r < n_req) ctx_off[r + 1] = carry + sh[threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 0) carry += sh[1023];
    __syncthreads();
  }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kThreads) void gather_pages_kernel(
    int n_req, const u32x4* __restrict__ kpool, const u32x4* __restrict__ vpool, int n_pages,
    const int32_t* __restrict__ page_table, int max_blocks, const int64_t* __restrict__ ctx_off,
    u32x4* __restrict__ kctx, u32x4* __restrict__ vctx, int64_t cap_pages, int page_vec /* 16-byte vectors per page */) {
  const int64_t total_pages = ctx_off[n_req] / SKV_BLOCK_TOKENS;
  for (int64_t p = blockIdx.x; p < total_pages; p += gridDim.x) {
    // request that owns output page p: last r with ctx_off[r]/16 <= p
    int lo = 0, hi = n_req;  // invariant: ctx_off[lo] <= 16p < ctx_off[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (ctx_off[mid] <= p * SKV_BLOCK_TOKENS) lo = mid; else hi = mid;
    }
    const int j = (int)(p - ctx_off[lo] / SKV_BLOCK_TOKENS);
    if (j >= max_blocks) continue;
    const int page = page_table[(size_t)lo * max_blocks + j];
    if (page < 0 || page >= n_pages || p >= cap_pages) continue;  // uniform per workgroup
    const u32x4* ks = kpool + (size_t)page * page_vec;
    const u32x4* vs = vpool + (size_t)page * page_vec;
    u32x4* kd = kctx + (size_t)p * page_vec;
    u32x4* vd = vctx + (size_t)p * page_vec;
    for (int base = 0; base < page_vec; base += kThreads * kUnroll) {
      u32x4 a[kUnroll], b[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int i = base + u * kThreads + threadIdx.x;
        if (i < page_vec) {
          a[u] = __builtin_nontemporal_load(ks + i);
          b[u] = __builtin_nontemporal_load(vs + i);
        }
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int i = base + u * kThreads + threadIdx.x;
        if (i < page_vec) {
          __builtin_nontemporal_store(a[u], kd + i);
          __builtin_nontemporal_store(b[u], vd + i);
        }
      }
    }
  }
}

// Inverse of the gather: one workgroup per (request, new block) slot of the table, persistent grid.
__global__ __launch_bounds__(kThreads) void scatter_pages_kernel(
    int n_req, const u32x4* __restrict__ knew, const u32x4* __restrict__ vnew, const int32_t* __restrict__ q_off,
    const int32_t* __restrict__ new_pages, int max_new_blocks, u32x4* __restrict__ kpool, u32x4* __restrict__ vpool,
    int n_pages, int page_vec) {
  const int64_t slots = (int64_t)n_req * max_new_blocks;
  for (int64_t sidx = blockIdx.x; sidx < slots; sidx += gridDim.x) {
    const int r = (int)(sidx / max_new_blocks), j = (int)(sidx % max_new_blocks);
    const int page = new_pages[sidx];
    const int qb = q_off[r];
    const int full = (q_off[r + 1] - qb) / SKV_BLOCK_TOKENS;
    if (page < 0 || page >= n_pages || j >= full) continue;  // uniform per workgroup
    const size_t src = ((size_t)qb + (size_t)j * SKV_BLOCK_TOKENS) * (page_vec / SKV_BLOCK_TOKENS);  // 16-byte vectors per row
    const u32x4* ks = knew + src;
    const u32x4* vs = vnew + src;
    u32x4* kd = kpool + (size_t)page * page_vec;
    u32x4* vd = vpool + (size_t)page * page_vec;
    for (int base = 0; base < page_vec; base += kThreads * kUnroll) {
      u32x4 a[kUnroll], b[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int i = base + u * kThreads + threadIdx.x;
        if (i < page_vec) {
          a[u] = __builtin_nontemporal_load(ks + i);
          b[u] = __builtin_nontemporal_load(vs + i);
        }
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int i = base + u * kThreads + threadIdx.x;
        if (i < page_vec) {
          __builtin_nontemporal_store(a[u], kd + i);
          __builtin_nontemporal_store(b[u], vd + i);
        }
      }
    }
  }
}

// Plain streaming copy, same vector width and loads-before-stores shape as the page copies above.
__global__ __launch_bounds__(kThreads) void stream_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                               int64_t n_vec) {
  const int64_t stride = (int64_t)gridDim.x * kThreads * kUnroll;
  for (int64_t base = (int64_t)blockIdx.x * kThreads * kUnroll; base < n_vec; base += stride) {
    u32x4 a[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t i = base + (int64_t)u * kThreads + threadIdx.x;
      if (i < n_vec) a[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t i = base + (int64_t)u * kThreads + threadIdx.x;
      if (i < n_vec) __builtin_nontemporal_store(a[u], dst + i);
    }
  }
}

}  // namespace

extern "C" int skv_stream_copy(void* d_dst, const void* d_src, size_t bytes, void* stream) {
  if (bytes == 0) return SKV_OK;
  if (!d_dst || !d_src || (bytes & 15) || (((uintptr_t)d_dst | (uintptr_t)d_src) & 15)) return SKV_EINVAL;
  const int64_t n_vec = (int64_t)(bytes / 16);
  const int64_t per_wg = (int64_t)kThreads * kUnroll;
  const int64_t want = (n_vec + per_wg - 1) / per_wg;
  stream_copy_kernel<<<(int)(want < 256 * 16 ? want : 256 * 16), kThreads, 0, (hipStream_t)stream>>>(
      (const u32x4*)d_src, (u32x4*)d_dst, n_vec);
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_scatter_kv(const skv_attn_desc* desc, int32_t n_req, const void* d_knew, const void* d_vnew,
                              const int32_t* d_q_off, const int32_t* d_new_pages, int32_t max_new_blocks,
                              void* d_kpool, void* d_vpool, int32_t n_pages, void* stream) {
  if (!desc || n_req < 0 || n_pages < 0 || max_new_blocks < 0) return SKV_EINVAL;
  if (desc->dtype != SKV_F32 && desc->dtype != SKV_BF16) return SKV_EINVAL;
  if (desc->n_kv_heads < 1 || desc->head_dim < 1) return SKV_EINVAL;
  const int64_t row_bytes = (int64_t)desc->n_kv_heads * desc->head_dim * (desc->dtype == SKV_F32 ? 4 : 2);
  if (row_bytes % 16 || row_bytes * SKV_BLOCK_TOKENS / 16 > 0x7fffffff) return SKV_EINVAL;
  if (n_req == 0 || max_new_blocks == 0) return SKV_OK;
  if (!d_knew || !d_vnew || !d_q_off || !d_new_pages || !d_kpool || !d_vpool) return SKV_EINVAL;
  if (((uintptr_t)d_kpool | (uintptr_t)d_vpool | (uintptr_t)d_knew | (uintptr_t)d_vnew) & 15) return SKV_EINVAL;
  const int64_t slots = (int64_t)n_req * max_new_blocks;
  const int grid = (int)(slots < 256 * 16 ? slots : 256 * 16);
  scatter_pages_kernel<<<grid, kThreads, 0, (hipStream_t)stream>>>(
      n_req, (const u32x4*)d_knew, (const u32x4*)d_vnew, d_q_off, d_new_pages, max_new_blocks, (u32x4*)d_kpool,
      (u32x4*)d_vpool, n_pages, (int)(row_bytes * SKV_BLOCK_TOKENS / 16));
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}

extern "C" int skv_gather_kv(const skv_attn_desc* desc, int32_t n_req, const void* d_kpool,
                             const void* d_vpool, int32_t n_pages, const int32_t* d_matched_len,
                             const int32_t* d_page_table, int32_t max_blocks, int64_t* d_ctx_off,
                             void* d_kctx, void* d_vctx, int64_t ctx_capacity_tokens, void* stream) {
  if (!desc || n_req < 0 || n_pages < 0 || max_blocks < 0 || ctx_capacity_tokens < 0) return SKV_EINVAL;
  if (desc->dtype != SKV_F32 && desc->dtype != SKV_BF16) return SKV_EINVAL;
  if (desc->n_kv_heads < 1 || desc->head_dim < 1) return SKV_EINVAL;
  const int64_t page_bytes = (int64_t)SKV_BLOCK_TOKENS * desc->n_kv_heads * desc->head_dim *
                             (desc->dtype == SKV_F32 ? 4 : 2);
  if (page_bytes % 16 || page_bytes / 16 > 0x7fffffff) return SKV_EINVAL;
  if (!d_ctx_off) return SKV_EINVAL;
  if (n_req > 0 && (!d_matched_len || !d_kpool || !d_vpool || !d_kctx || !d_vctx)) return SKV_EINVAL;
  if (n_req > 0 && max_blocks > 0 && !d_page_table) return SKV_EINVAL;
  if (((uintptr_t)d_kpool | (uintptr_t)d_vpool | (uintptr_t)d_kctx | (uintptr_t)d_vctx) & 15) return SKV_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  ctx_offsets_kernel<<<1, 1024, 0, st>>>(n_req, d_matched_len, d_ctx_off);
  SKV_HIP(hipGetLastError());
  if (n_req == 0 || max_blocks == 0) return SKV_OK;
  int64_t upper = (int64_t)n_req * max_blocks;  // pages the batch can reference at most
  int grid = (int)(upper < 256 * 16 ? upper : 256 * 16);
  gather_pages_kernel<<<grid, kThreads, 0, st>>>(
      n_req, (const u32x4*)d_kpool, (const u32x4*)d_vpool, n_pages, d_page_table, max_blocks, d_ctx_off,
      (u32x4*)d_kctx, (u32x4*)d_vctx, ctx_capacity_tokens / SKV_BLOCK_TOKENS, (int)(page_bytes / 16));
  SKV_HIP(hipGetLastError());
  return SKV_OK;
}
