// KV hand-off and KV append: byte copies from contiguous per-token K,V rows
// into the paged cache [num_blocks, n, 16, s].  HBM-bound; every lane moves
// 16-byte pieces, reads are 2*s-byte runs (one head of one token), writes are
// contiguous runs of a whole (page, head-group).
#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kPage = 16;          // tokens per page
constexpr int kMigThreads = 256;
constexpr int kMigPer = 20;        // 16-byte pieces per thread

// One workgroup moves HG = 20 (s = 128) or 40 (s = 64) heads of one page of K or of V: 80 KB in, 80 KB out,
// twenty 16-byte pieces per thread.  What the kernel is built around, measured on this chip with the source
// not resident in any cache (the hand-off runs long after the projection that wrote it):
//  * A hand-off of a few thousand tokens is one wave of memory latency, not a stream: all of a thread's loads
//    are issued back to back before anything waits, the block id is requested together with them (it is only
//    needed for the stores), and the common case - a full page, a full head group - runs without a single
//    predicate, because per-load predicates made the compiler wait for every load before issuing the next.
//  * The source is read exactly once: non-temporal loads (no allocation in L2 / last-level cache) moved the
//    16 k-token hand-off from 4.9 to 6.1 TB/s.  Non-temporal stores cost more than they save.
//  * Stores are paced: at most two in flight per wave.  With every wave pushing all its stores at once the
//    same copy took 1.5-2 us longer at 2 k tokens (write bursts back up into the read path).
// grid: x = logical page index within the sequence, y = sequence, z = 2 * head_group + (0: K, 1: V)
template <int HD>
__global__ __launch_bounds__(kMigThreads) void kv_migrate_kernel(
    const uint16_t* __restrict__ k_src, const uint16_t* __restrict__ v_src,
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ block_tables, int max_blocks,
    uint16_t* __restrict__ k_cache, uint16_t* __restrict__ v_cache, int n_heads) {
  constexpr int CPS = HD / 8;                                 // 16-byte pieces per (token, head) row
  constexpr int HG = kMigPer * kMigThreads / (kPage * CPS);   // heads per workgroup
  static_assert(HG * kPage * CPS == kMigPer * kMigThreads, "whole rounds of pieces");
  const int lb = blockIdx.x;
  const int seq = blockIdx.y;
  const int which = blockIdx.z & 1;
  const int head0 = (blockIdx.z >> 1) * HG;
  const int32_t* blk_ptr = block_tables + (size_t)seq * max_blocks + lb;
  const int start = cu_seqlens[seq];
  const int len = cu_seqlens[seq + 1] - start;
  const int tok0 = lb * kPage;
  if (tok0 >= len) return;
  const int ntok = min(kPage, len - tok0);
  const int h = n_heads * HD;
  const int heads = min(HG, n_heads - head0);
  const uint16_t* src = (which ? v_src : k_src) + ((size_t)start + tok0) * h + (size_t)head0 * HD;
  uint16_t* cache = which ? v_cache : k_cache;
  // piece c of the workgroup: head c / (16 CPS), slot (c / CPS) % 16, 16-byte piece c % CPS of that row;
  // the destination of piece c is simply byte 16 c of the (page, head group) run
  u32x4 buf[kMigPer];
  if (ntok == kPage && heads == HG) {
#pragma unroll
    for (int u = 0; u < kMigPer; ++u) {
      const int c = threadIdx.x + u * kMigThreads;
      const int ch = c % CPS, slot = (c / CPS) % kPage, hd = c / (CPS * kPage);
      buf[u] = __builtin_nontemporal_load(
          reinterpret_cast<const u32x4*>(src + (size_t)slot * h + hd * HD + ch * 8));
    }
    __builtin_amdgcn_sched_barrier(0);  // the block id is not waited for before the loads above are out
    const int blk = *blk_ptr;
    uint16_t* dst = cache + ((size_t)blk * n_heads + head0) * (size_t)(kPage * HD);
    __builtin_amdgcn_s_waitcnt(0x0070 | (0xf << 8));  // vmcnt(0): every load has landed
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < kMigPer; ++u) {
      st16(dst + (size_t)(threadIdx.x + u * kMigThreads) * 8, buf[u]);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(0x0071 | (0xf << 8));  // vmcnt(1): at most two stores in flight
      __builtin_amdgcn_sched_barrier(0);
    }
    return;
  }
  // Ragged page (the sequence ends inside it) or a narrower head group (the last one; every one of a model with
  // fewer key/value heads than HG): the same two phases over the rounds that hold a real head, with the row
  // and head indices of the loads clamped into the page (a harmless re-read) and the stores predicated.
  const int rounds = min(kMigPer, (heads * kPage * CPS + kMigThreads - 1) / kMigThreads);
  u32x4 rag[kMigPer];  // (an array of its own: sharing `buf` made the compiler re-plan the path above)
#pragma unroll
  for (int u = 0; u < kMigPer; ++u) {
    const int c = threadIdx.x + u * kMigThreads;
    const int ch = c % CPS, slot = min((c / CPS) % kPage, ntok - 1), hd = min(c / (CPS * kPage), heads - 1);
    if (u < rounds)  // uniform
      rag[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (size_t)slot * h + hd * HD + ch * 8));
  }
  __builtin_amdgcn_sched_barrier(0);
  const int blk = *blk_ptr;
  uint16_t* dst = cache + ((size_t)blk * n_heads + head0) * (size_t)(kPage * HD);
#pragma unroll
  for (int u = 0; u < kMigPer; ++u) {
    const int c = threadIdx.x + u * kMigThreads;
    const int slot = (c / CPS) % kPage, hd = c / (CPS * kPage);
    if (u < rounds && slot < ntok && hd < heads) st16(dst + (size_t)c * 8, rag[u]);
  }
}

hipError_t launch_kv_migrate(const void* k_src, const void* v_src, const int32_t* cu_seqlens, int B,
                             int max_seqlen, const int32_t* block_tables, int max_blocks, void* k_cache,
                             void* v_cache, int n_heads, int head_dim, hipStream_t stream) {
  const int pages = (max_seqlen + kPage - 1) / kPage;
  if (pages <= 0 || B <= 0) return hipSuccess;
  if (head_dim != 64 && head_dim != 128) return hipErrorInvalidValue;
  if (pages > max_blocks) return hipErrorInvalidValue;  // the kernel reads block_tables[seq][page] for every page
  const int hg = kMigPer * kMigThreads / (kPage * (head_dim / 8));
  const int groups = (n_heads + hg - 1) / hg;
  if (B > 65535 || 2 * groups > 65535) return hipErrorInvalidValue;
  const dim3 grid(pages, B, 2 * groups);
  if (head_dim == 128)
    hipLaunchKernelGGL(kv_migrate_kernel<128>, grid, dim3(kMigThreads), 0, stream, (const uint16_t*)k_src,
                       (const uint16_t*)v_src, cu_seqlens, block_tables, max_blocks, (uint16_t*)k_cache,
                       (uint16_t*)v_cache, n_heads);
  else
    hipLaunchKernelGGL(kv_migrate_kernel<64>, grid, dim3(kMigThreads), 0, stream, (const uint16_t*)k_src,
                       (const uint16_t*)v_src, cu_seqlens, block_tables, max_blocks, (uint16_t*)k_cache,
                       (uint16_t*)v_cache, n_heads);
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
