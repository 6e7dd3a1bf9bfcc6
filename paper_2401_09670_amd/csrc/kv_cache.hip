// KV hand-off and KV append: byte copies from contiguous per-token K,V rows
// into the paged cache [num_blocks, n, 16, s].  HBM-bound; every lane moves
// 16-byte pieces, reads are 2*s-byte runs (one head of one token), writes are
// contiguous runs of a whole (page, head-group).
#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kPage = 16;          // tokens per page
constexpr int kMigThreads = 256;
constexpr int kMigHeadsPerWg = 4;  // heads one workgroup moves for one page
constexpr int kMigUnroll = 4;

// grid: x = logical page index within the sequence, y = sequence,
//       z = 2 * head_group + (0: K, 1: V)
__global__ __launch_bounds__(kMigThreads) void kv_migrate_kernel(
    const uint16_t* __restrict__ k_src, const uint16_t* __restrict__ v_src,
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ block_tables, int max_blocks,
    uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache, int n_heads, int head_dim) {
  const int lb = blockIdx.x;
  const int seq = blockIdx.y;
  const int which = blockIdx.z & 1;
  const int head0 = (blockIdx.z >> 1) * kMigHeadsPerWg;
  const int start = cu_seqlens[seq];
  const int len = cu_seqlens[seq + 1] - start;
  const int tok0 = lb * kPage;
  if (tok0 >= len) return;
  const int ntok = min(kPage, len - tok0);
  const int blk = block_tables[(size_t)seq * max_blocks + lb];
  const int h = n_heads * head_dim;
  const int cps = head_dim >> 3;  // 16-byte chunks per (token, head) row
  const int heads = min(kMigHeadsPerWg, n_heads - head0);
  const int chunks = heads * kPage * cps;

  const uint16_t* src = (which ? v_src : k_src) + ((size_t)start + tok0) * h + (size_t)head0 * head_dim;
  uint16_t* dst = (which ? v_cache : k_cache) + ((size_t)blk * n_heads + head0) * (size_t)(kPage * head_dim);

  for (int base = threadIdx.x; base < chunks; base += kMigThreads * kMigUnroll) {
    u32x4 buf[kMigUnroll];
    bool ok[kMigUnroll];
#pragma unroll
    for (int u = 0; u < kMigUnroll; ++u) {
      const int c = base + u * kMigThreads;
      const int ch = c % cps;
      const int slot = (c / cps) % kPage;
      const int hd = c / (cps * kPage);
      ok[u] = (c < chunks) && (slot < ntok);
      if (ok[u]) buf[u] = ld16(src + (size_t)slot * h + hd * head_dim + ch * 8);
    }
#pragma unroll
    for (int u = 0; u < kMigUnroll; ++u) {
      const int c = base + u * kMigThreads;
      if (ok[u]) st16(dst + (size_t)c * 8, buf[u]);
    }
  }
}

hipError_t launch_kv_migrate(const void* k_src, const void* v_src, const int32_t* cu_seqlens, int B,
                             int max_seqlen, const int32_t* block_tables, int max_blocks, void* k_cache,
                             void* v_cache, int n_heads, int head_dim, hipStream_t stream) {
  const int pages = (max_seqlen + kPage - 1) / kPage;
  const int groups = (n_heads + kMigHeadsPerWg - 1) / kMigHeadsPerWg;
  if (pages <= 0 || B <= 0) return hipSuccess;
  if (B > 65535 || 2 * groups > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kv_migrate_kernel, dim3(pages, B, 2 * groups), dim3(kMigThreads), 0, stream,
                     (const uint16_t*)k_src, (const uint16_t*)v_src, cu_seqlens, block_tables, max_blocks,
                     (uint16_t*)k_cache, (uint16_t*)v_cache, n_heads, head_dim);
  return hipGetLastError();
}

// grid: x = sequence, y = 0: K, 1: V.  One row of n*s elements per workgroup.
__global__ __launch_bounds__(256) void kv_append_kernel(const uint16_t* __restrict__ k_new,
                                                        const uint16_t* __restrict__ v_new, int src_stride,
                                                        const int32_t* __restrict__ ctx_lens,
                                                        const int32_t* __restrict__ block_tables,
                                                        int max_blocks, uint16_t* __restrict__ k_cache,
                                                        uint16_t* __restrict__ v_cache, int n_heads,
                                                        int head_dim) {
  const int seq = blockIdx.x;
  const int which = blockIdx.y;
  const int pos = ctx_lens[seq];
  const int blk = block_tables[(size_t)seq * max_blocks + pos / kPage];
  const int slot = pos % kPage;
  const int cps = head_dim >> 3;
  const uint16_t* src = (which ? v_new : k_new) + (size_t)seq * src_stride;
  uint16_t* dst = (which ? v_cache : k_cache) + (size_t)blk * n_heads * (kPage * head_dim) +
                  (size_t)slot * head_dim;
  const int chunks = n_heads * cps;
  for (int c = threadIdx.x; c < chunks; c += 256) {
    const int hd = c / cps, ch = c % cps;
    st16(dst + (size_t)hd * (kPage * head_dim) + ch * 8, ld16(src + hd * head_dim + ch * 8));
  }
}

hipError_t launch_kv_append(const void* k_new, const void* v_new, int src_stride, const int32_t* ctx_lens,
                            const int32_t* block_tables, int B, int max_blocks, void* k_cache, void* v_cache,
                            int n_heads, int head_dim, hipStream_t stream) {
  if (B <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_append_kernel, dim3(B, 2), dim3(256), 0, stream, (const uint16_t*)k_new,
                     (const uint16_t*)v_new, src_stride, ctx_lens, block_tables, max_blocks,
                     (uint16_t*)k_cache, (uint16_t*)v_cache, n_heads, head_dim);
  return hipGetLastError();
}

}  // namespace ds
