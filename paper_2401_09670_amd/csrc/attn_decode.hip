// Decode attention over the paged KV cache: one query per (sequence, head).
// HBM-bound: the kernel's job is to stream each (page, head) run of K and V
// (16 tokens x s elements, contiguous) exactly once with 16-byte loads.
//
// grid = (heads, sequences, splits).  A workgroup of 4 waves takes one split
// of the sequence's pages; wave w takes pages w, w+4, ... of that split.  In
// a wave, s/8 lanes cover one token row (8 elements each), so one load
// instruction covers 64/(s/8) tokens.  Scores are reduced across the lanes
// of a token with xor-shuffles, softmax runs online in fp32, and the four
// waves' (max, sum, acc) states are merged through LDS.  With one split the
// result is written as bf16; with several, fp32 partial states go to the
// workspace and a second kernel merges them (fixed order: deterministic).
#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = 4;
constexpr int kDecPage = 16;

// 8-element bf16 dot product in fp32.  (Plain unpack + FMA: the packed bf16
// dot builtin was observed to be selected with repeated source registers by
// this compiler, giving wrong sums.)
__device__ __forceinline__ float dot8(const u32x4 a, const u32x4 b) {
  float acc = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    acc += bf16_lo(a[j]) * bf16_lo(b[j]);
    acc += bf16_hi(a[j]) * bf16_hi(b[j]);
  }
  return acc;
}

// partial state layout in the workspace, per (seq, head, split): [0]=max, [1]=sum, [2..2+HD) = acc
template <int HD>
__global__ __launch_bounds__(kDecThreads) void decode_attention_kernel(
    const uint16_t* __restrict__ q, int q_stride, const int32_t* __restrict__ kv_lens, int kv_len_add,
    const int32_t* __restrict__ block_tables, int max_blocks, const uint16_t* __restrict__ k_cache,
    const uint16_t* __restrict__ v_cache, int n_heads, int n_kv_heads, int pages_per_split, float scale_log2e,
    uint16_t* __restrict__ o, float* __restrict__ partial) {
  constexpr int LPT = HD / 8;          // lanes per token row
  constexpr int TPL = 64 / LPT;        // tokens per load instruction
  constexpr int NL = kDecPage / TPL;   // load instructions per page
  __shared__ float sm_m[kDecWaves], sm_l[kDecWaves];
  __shared__ float sm_acc[kDecWaves][HD];

  // Query heads that share a key/value head are n_kv_heads apart in launch order: with n_kv_heads a
  // multiple of 8 they land on the same chip partition at about the same time, so the group's K/V
  // pages come out of that partition's L2 after the first reader.  (Plain identity for n_kv = n.)
  const int kv_group = n_heads / n_kv_heads;
  const int kv_head = blockIdx.x % n_kv_heads;
  const int head = kv_head * kv_group + blockIdx.x / n_kv_heads;
  const int seq = blockIdx.y, split = blockIdx.z;
  const int n_splits = gridDim.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tg = lane / LPT, dc = lane % LPT;

  const int kv_len = kv_lens[seq] + kv_len_add;
  const int n_pages = (kv_len + kDecPage - 1) / kDecPage;
  const int page_lo = split * pages_per_split;
  const int page_hi = min(n_pages, page_lo + pages_per_split);

  const u32x4 qv = ld16(q + (size_t)seq * q_stride + head * HD + dc * 8);
  const int32_t* bt = block_tables + (size_t)seq * max_blocks;
  const size_t page_elems = (size_t)kDecPage * HD;

  float m_run = -INFINITY, l_run = 0.f;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;

  // Software pipeline over this wave's pages: the block id is fetched two pages ahead and the K/V
  // rows one page ahead, so neither the table lookup nor the HBM latency sits between two pages.
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const size_t lane_off = (size_t)tg * HD + dc * 8;
  auto fetch = [&](int blk, u32x4* kd, u32x4* vd) {
    const size_t base = ((size_t)blk * n_kv_heads + kv_head) * page_elems + lane_off;
#pragma unroll
    for (int j = 0; j < NL; ++j) kd[j] = ld16(k_cache + base + (size_t)j * TPL * HD);
#pragma unroll
    for (int j = 0; j < NL; ++j) vd[j] = ld16(v_cache + base + (size_t)j * TPL * HD);
  };
  u32x4 kr[NL], vr[NL], kn[NL], vn[NL];
#pragma unroll
  for (int j = 0; j < NL; ++j) kr[j] = vr[j] = kn[j] = vn[j] = u32x4{0, 0, 0, 0};
  const int pg0 = page_lo + wave_u;
  int blk1 = 0, blk2 = 0;  // block ids of the pages one and two steps ahead of `pg`
  if (pg0 < page_hi) fetch(bt[pg0], kr, vr);
  if (pg0 + kDecWaves < page_hi) blk1 = bt[pg0 + kDecWaves];
  if (pg0 + 2 * kDecWaves < page_hi) blk2 = bt[pg0 + 2 * kDecWaves];

  for (int pg = pg0; pg < page_hi; pg += kDecWaves) {
    if (pg + kDecWaves < page_hi) fetch(blk1, kn, vn);
    blk1 = blk2;
    if (pg + 3 * kDecWaves < page_hi) blk2 = bt[pg + 3 * kDecWaves];

    float sc[NL];
    float tmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      float d = dot8(qv, kr[j]);
#pragma unroll
      for (int off = 1; off < LPT; off <<= 1) d += __shfl_xor(d, off, 64);
      const int tok = pg * kDecPage + j * TPL + tg;
      sc[j] = (tok < kv_len) ? d : -INFINITY;
      tmax = fmaxf(tmax, sc[j]);
    }
#pragma unroll
    for (int off = LPT; off < 64; off <<= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, off, 64));
    // the first token of a visited page is always < kv_len, so tmax is finite
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = exp2f((m_run - m_new) * scale_log2e);
    const float mb = m_new * scale_log2e;
    l_run *= alpha;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] *= alpha;
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      const float p = exp2f(sc[j] * scale_log2e - mb);
      l_run += p;
      // Slots past the sequence's end hold whatever the pool's memory held before (possibly NaN or Inf bit
      // patterns): their weight is 0, but 0 * NaN is NaN, so their V bits are cleared as well.
      const uint32_t keep = (pg * kDecPage + j * TPL + tg < kv_len) ? 0xffffffffu : 0u;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t v2 = vr[j][e] & keep;
        acc[2 * e] += p * bf16_lo(v2);
        acc[2 * e + 1] += p * bf16_hi(v2);
      }
    }
    m_run = m_new;
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      kr[j] = kn[j];
      vr[j] = vn[j];
    }
  }

  // merge the token groups of the wave: every lane of a group carries the same l_run
#pragma unroll
  for (int off = LPT; off < 64; off <<= 1) {
    l_run += __shfl_xor(l_run, off, 64);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += __shfl_xor(acc[j], off, 64);
  }
  if (lane < LPT) {
#pragma unroll
    for (int j = 0; j < 8; ++j) sm_acc[wave][lane * 8 + j] = acc[j];
    if (lane == 0) {
      sm_m[wave] = m_run;
      sm_l[wave] = l_run;
    }
  }
  __syncthreads();
  // merge the waves (a wave that saw no page has max = -inf, sum = 0 and weight 0)
  if (tid < HD) {
    float m = sm_m[0];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) m = fmaxf(m, sm_m[w]);
    float l = 0.f, a = 0.f;
    if (m > -INFINITY) {
#pragma unroll
      for (int w = 0; w < kDecWaves; ++w) {
        const float f = exp2f((sm_m[w] - m) * scale_log2e);
        l += sm_l[w] * f;
        a += sm_acc[w][tid] * f;
      }
    }
    if (n_splits == 1) {
      reinterpret_cast<__bf16*>(o)[((size_t)seq * n_heads + head) * HD + tid] = (__bf16)(a / l);
    } else {
      float* dst = partial + (((size_t)seq * n_heads + head) * n_splits + split) * (HD + 2);
      if (tid == 0) {
        dst[0] = m;
        dst[1] = l;
      }
      dst[2 + tid] = a;
    }
  }
}

template <int HD>
__global__ __launch_bounds__(HD) void decode_combine_kernel(const float* __restrict__ partial, int n_splits,
                                                            float scale_log2e, uint16_t* __restrict__ o) {
  const size_t item = blockIdx.x;  // seq * n_heads + head
  const float* src = partial + item * n_splits * (HD + 2);
  const int tid = threadIdx.x;
  float m = -INFINITY;
  for (int s = 0; s < n_splits; ++s) m = fmaxf(m, src[s * (HD + 2)]);
  float l = 0.f, a = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float ms = src[s * (HD + 2)];
    if (ms > -INFINITY) {
      const float f = exp2f((ms - m) * scale_log2e);
      l += src[s * (HD + 2) + 1] * f;
      a += src[s * (HD + 2) + 2 + tid] * f;
    }
  }
  reinterpret_cast<__bf16*>(o)[item * HD + tid] = (__bf16)(a / l);
}

// Enough workgroups to cover the chip about twice, but never less than 8 pages per split.
int decode_attention_splits(int B, int n_heads, int max_kv_len) {
  const int pages = (max_kv_len + kDecPage - 1) / kDecPage;
  const long items = (long)B * n_heads;
  int splits = (int)((2 * 256 + items - 1) / items);
  const int max_splits = (pages + 2 * kDecWaves - 1) / (2 * kDecWaves);
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  return splits;
}

size_t decode_attention_workspace_bytes(int B, int n_heads, int head_dim, int max_kv_len) {
  const int splits = decode_attention_splits(B, n_heads, max_kv_len);
  if (splits == 1) return 0;
  return (size_t)B * n_heads * splits * (head_dim + 2) * sizeof(float);
}

hipError_t launch_decode_attention(const void* q, int q_stride, const int32_t* kv_lens, int kv_len_add,
                                   const int32_t* block_tables, int B, int max_blocks, int max_kv_len,
                                   const void* k_cache, const void* v_cache, int n_heads, int n_kv_heads,
                                   int head_dim, void* o, void* workspace, hipStream_t stream) {
  if (B <= 0) return hipSuccess;
  if (n_kv_heads <= 0 || n_heads % n_kv_heads != 0) return hipErrorInvalidValue;
  if (B > 65535) return hipErrorInvalidValue;
  const int splits = decode_attention_splits(B, n_heads, max_kv_len);
  const int pages = (max_kv_len + kDecPage - 1) / kDecPage;
  const int pps = (pages + splits - 1) / splits;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
  const dim3 grid(n_heads, B, splits);
  if (head_dim == 128) {
    hipLaunchKernelGGL(decode_attention_kernel<128>, grid, dim3(kDecThreads), 0, stream, (const uint16_t*)q,
                       q_stride, kv_lens, kv_len_add, block_tables, max_blocks, (const uint16_t*)k_cache,
                       (const uint16_t*)v_cache, n_heads, n_kv_heads, pps, scale_log2e, (uint16_t*)o, (float*)workspace);
    if (splits > 1)
      hipLaunchKernelGGL(decode_combine_kernel<128>, dim3(B * n_heads), dim3(128), 0, stream,
                         (const float*)workspace, splits, scale_log2e, (uint16_t*)o);
  } else if (head_dim == 64) {
    hipLaunchKernelGGL(decode_attention_kernel<64>, grid, dim3(kDecThreads), 0, stream, (const uint16_t*)q,
                       q_stride, kv_lens, kv_len_add, block_tables, max_blocks, (const uint16_t*)k_cache,
                       (const uint16_t*)v_cache, n_heads, n_kv_heads, pps, scale_log2e, (uint16_t*)o, (float*)workspace);
    if (splits > 1)
      hipLaunchKernelGGL(decode_combine_kernel<64>, dim3(B * n_heads), dim3(64), 0, stream,
                         (const float*)workspace, splits, scale_log2e, (uint16_t*)o);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ds
