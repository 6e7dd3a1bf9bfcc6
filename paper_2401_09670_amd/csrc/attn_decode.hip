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

// A K/V row is read once per decoding step and the cache of a batch is far larger than the last-level cache,
// so the loads are non-temporal (no allocation on the way in): 131 -> 117.5 us per step at OPT-13B, batch 64,
// context 512-576, i.e. 5.5 -> 6.1 TB/s.
__device__ __forceinline__ u32x4 ld16_kv(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
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
    for (int j = 0; j < NL; ++j) kd[j] = ld16_kv(k_cache + base + (size_t)j * TPL * HD);
#pragma unroll
    for (int j = 0; j < NL; ++j) vd[j] = ld16_kv(v_cache + base + (size_t)j * TPL * HD);
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
      reinterpret_cast<__bf16*>(o)[((size_t)seq * n_heads + head) * HD + tid] = (__bf16)(l > 0.f ? a / l : 0.f);  // no key at all (kv_len = 0): defined as 0
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
  reinterpret_cast<__bf16*>(o)[item * HD + tid] = (__bf16)(l > 0.f ? a / l : 0.f);  // no key at all (kv_len = 0): defined as 0
}

// ---------------------------------------------------------------------------------------------
// Grouped-query form (n_kv_heads < n_heads, head size 128, up to 16 query heads per key/value head).
// The kernel above would stream a key/value head's pages once per query head of its group (out of L2
// after the first, but through the same load path); here one workgroup serves the whole group, so
// every page is read once, and the group's heads ride along as the second dimension of 16x16x32
// matrix-core tiles:
//   scores  S[key, head]   = K[key, :] . Q[head, :]      A = K rows (16 keys), B = Q rows (16 heads, zero padded)
//   output  O^T[d, head]  += V^T[d, key] . P[key, head]   A = V^T (16 d), B = P in the registers S came out in
// grid = (n_kv_heads, sequences, splits); a wave takes two pages (32 keys = one depth of the second
// product) per iteration: pairs wave, wave + 4, ... of its split.  In the tile result layout a lane holds
// one head (lane % 16) and keys 4g .. 4g+3 of each page (g = lane / 16), so the running max / sum /
// rescale factor of the online softmax are per-lane scalars once the maximum has been exchanged between
// the four lane groups, and the probabilities are already in place as operand B of the second product if
// its depth index is read as (g, page, key % 4).  V has to supply the same depth order with d along the
// rows: the two V pages go through a wave-private, padded LDS area and come back as 2-byte reads (the
// kernel is HBM-bound with a wide margin: 16 matrix instructions per 16 KB of K and V).
// Partial states per (sequence, head, split) use the layout of the kernel above, so the same combine
// kernel finishes split launches.
// ---------------------------------------------------------------------------------------------
constexpr int kGqaHD = 128;
constexpr int kGqaVRow = kGqaHD + 8;  // LDS row of a staged V page in elements: 272 bytes (16-byte aligned), so
                                      // the four lane groups' rows (4 rows apart) start 64 bytes apart in the banks

__global__ __launch_bounds__(kDecThreads) __attribute__((amdgpu_waves_per_eu(2))) void decode_attention_gqa_kernel(
    const uint16_t* __restrict__ q, int q_stride, const int32_t* __restrict__ kv_lens, int kv_len_add,
    const int32_t* __restrict__ block_tables, int max_blocks, const uint16_t* __restrict__ k_cache,
    const uint16_t* __restrict__ v_cache, int n_heads, int n_kv_heads, int pages_per_split, float scale_log2e,
    uint16_t* __restrict__ o, float* __restrict__ partial) {
  constexpr int HD = kGqaHD;
  constexpr int kStage = 2 * kDecPage * kGqaVRow;            // elements of one wave's V staging area
  constexpr int kMergeFloats = kDecWaves * 16 * (HD + 2);    // [wave][head][max, sum, acc[HD]]
  constexpr int kLdsBytes = kDecWaves * kStage * 2 > kMergeFloats * 4 ? kDecWaves * kStage * 2 : kMergeFloats * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kLdsBytes];

  const int G = n_heads / n_kv_heads;  // 2..16 query heads share this key/value head
  const int kv_head = blockIdx.x, seq = blockIdx.y, split = blockIdx.z;
  const int n_splits = gridDim.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hl = lane & 15, g = lane >> 4;  // head (or key, or d) index inside a tile; lane group

  const int kv_len = kv_lens[seq] + kv_len_add;
  const int n_pages = (kv_len + kDecPage - 1) / kDecPage;
  const int page_lo = split * pages_per_split;
  const int page_hi = min(n_pages, page_lo + pages_per_split);
  const int32_t* bt = block_tables + (size_t)seq * max_blocks;
  const size_t page_elems = (size_t)kDecPage * HD;

  // operand B of the score product: Q[head = hl][32 s + 8 g .. + 8), zero rows for hl >= G
  u32x4 qf[4];
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4) {
    qf[s4] = u32x4{0, 0, 0, 0};
    if (hl < G) qf[s4] = ld16(q + (size_t)seq * q_stride + (size_t)(kv_head * G + hl) * HD + 32 * s4 + 8 * g);
  }

  floatx4 acc[HD / 16];  // O^T[d = 16 db + 4 g + r][head = hl]
#pragma unroll
  for (int db = 0; db < HD / 16; ++db) acc[db] = floatx4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;  // l_run: this lane group's share of the sum

  uint16_t* vst = reinterpret_cast<uint16_t*>(smem) + wave * kStage;
  // K as operand A: lane (key = hl, group g) holds K[key][32 s + 8 g .. + 8) for s = 0..3.
  // V rows as they lie in the page: load i of a page covers rows 4 i .. 4 i + 3, lane -> row 4 i + lane / 16,
  // 16-byte piece lane % 16.
  auto fetch = [&](int blk0, int blk1, u32x4* kd, u32x4* vd) {
    const size_t b0 = ((size_t)blk0 * n_kv_heads + kv_head) * page_elems;
    const size_t b1 = ((size_t)blk1 * n_kv_heads + kv_head) * page_elems;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      kd[s4] = ld16_kv(k_cache + b0 + hl * HD + 32 * s4 + 8 * g);
      kd[4 + s4] = ld16_kv(k_cache + b1 + hl * HD + 32 * s4 + 8 * g);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      vd[i] = ld16_kv(v_cache + b0 + (size_t)(4 * i + g) * HD + hl * 8);
      vd[4 + i] = ld16_kv(v_cache + b1 + (size_t)(4 * i + g) * HD + hl * 8);
    }
  };
  // block ids of pair `pg` (second page clamped to the first where the sequence ends on an odd page: its
  // keys are masked, the loads just stay inside the pool)
  auto ids = [&](int pg, int& b0, int& b1) {
    b0 = bt[pg];
    b1 = pg + 1 < page_hi ? bt[pg + 1] : b0;
  };

  u32x4 kr[8], vr[8], kn[8], vn[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) kr[j] = vr[j] = kn[j] = vn[j] = u32x4{0, 0, 0, 0};
  constexpr int kStep = 2 * kDecWaves;  // pages between two pairs of one wave
  const int pg0 = page_lo + 2 * wave;
  int nb0 = 0, nb1 = 0;
  if (pg0 < page_hi) {
    int b0, b1;
    ids(pg0, b0, b1);
    fetch(b0, b1, kr, vr);
  }
  if (pg0 + kStep < page_hi) ids(pg0 + kStep, nb0, nb1);

  for (int pg = pg0; pg < page_hi; pg += kStep) {
    if (pg + kStep < page_hi) fetch(nb0, nb1, kn, vn);
    if (pg + 2 * kStep < page_hi) ids(pg + 2 * kStep, nb0, nb1);

    // scores of 32 keys x 16 heads
    floatx4 s0 = floatx4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[s4]),
                                                   __builtin_bit_cast(bf16x8, qf[s4]), s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[4 + s4]),
                                                   __builtin_bit_cast(bf16x8, qf[s4]), s1, 0, 0, 0);
    }
    // this lane: head hl, keys pg*16 + 4g + r (s0) and (pg+1)*16 + 4g + r (s1).  The second page counts only
    // if it belongs to this split (the next split, if any, starts with it otherwise).
    const int key0 = pg * kDecPage + 4 * g;
    const int end1 = pg + 1 < page_hi ? kv_len : 0;  // keys of the second page are valid below this
    float sc[8];
    float tmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      sc[r] = key0 + r < kv_len ? s0[r] : -INFINITY;
      sc[4 + r] = key0 + kDecPage + r < end1 ? s1[r] : -INFINITY;
      tmax = fmaxf(tmax, fmaxf(sc[r], sc[4 + r]));
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    // the first key of a visited pair is always < kv_len, so tmax is finite
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = exp2f((m_run - m_new) * scale_log2e);
    const float mb = m_new * scale_log2e;
    float pr[8];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      pr[j] = exp2f(sc[j] * scale_log2e - mb);
      psum += pr[j];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < HD / 16; ++db) acc[db] *= alpha;
    u32x4 pf;  // depth index 8 g + j  <->  (page j / 4, key 4 g + j % 4)
    pf[0] = pack_bf16(pr[0], pr[1]);
    pf[1] = pack_bf16(pr[2], pr[3]);
    pf[2] = pack_bf16(pr[4], pr[5]);
    pf[3] = pack_bf16(pr[6], pr[7]);

    // stage the two V pages; rows past the sequence's end are written as zeros (what the pool holds there
    // may be NaN or Inf bit patterns, and 0 * NaN is NaN)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 4 * i + g;
      const u32x4 z = u32x4{0, 0, 0, 0};
      const u32x4 v0 = pg * kDecPage + row < kv_len ? vr[i] : z;
      const u32x4 v1 = (pg + 1) * kDecPage + row < end1 ? vr[4 + i] : z;
      *reinterpret_cast<u32x4*>(vst + row * kGqaVRow + hl * 8) = v0;
      *reinterpret_cast<u32x4*>(vst + (kDecPage + row) * kGqaVRow + hl * 8) = v1;
    }
    // operand A of the second product for d block db: V[(page, key 4g + r)][16 db + hl] in depth order
#pragma unroll
    for (int db = 0; db < HD / 16; ++db) {
      const uint16_t* col = vst + (4 * g) * kGqaVRow + 16 * db + hl;
      u32x4 vf;
#pragma unroll
      for (int pgi = 0; pgi < 2; ++pgi) {
        const uint16_t* c2 = col + pgi * kDecPage * kGqaVRow;
        vf[2 * pgi] = (uint32_t)c2[0] | ((uint32_t)c2[kGqaVRow] << 16);
        vf[2 * pgi + 1] = (uint32_t)c2[2 * kGqaVRow] | ((uint32_t)c2[3 * kGqaVRow] << 16);
      }
      acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf),
                                                        __builtin_bit_cast(bf16x8, pf), acc[db], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      kr[j] = kn[j];
      vr[j] = vn[j];
    }
  }

  // the four lane groups' shares of the sum
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  __syncthreads();  // every wave is done with its staging area: the merge area overlays it
  float* mg = reinterpret_cast<float*>(smem);  // [wave][head][max, sum, acc[HD]]
  {
    float* dst = mg + (size_t)(wave * 16 + hl) * (HD + 2);
    if (g == 0) {
      dst[0] = m_run;
      dst[1] = l_run;
    }
#pragma unroll
    for (int db = 0; db < HD / 16; ++db)
#pragma unroll
      for (int r = 0; r < 4; ++r) dst[2 + 16 * db + 4 * g + r] = acc[db][r];
  }
  __syncthreads();
  // thread -> head tid / 16, d = 8 (tid % 16) .. + 8; a wave that saw no pair has max = -inf and weight 0
  const int h = tid >> 4, d0 = (tid & 15) * 8;
  if (h < G) {
    float m = -INFINITY;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) m = fmaxf(m, mg[(size_t)(w * 16 + h) * (HD + 2)]);
    float l = 0.f, a[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) a[j] = 0.f;
    if (m > -INFINITY) {
#pragma unroll
      for (int w = 0; w < kDecWaves; ++w) {
        const float* src = mg + (size_t)(w * 16 + h) * (HD + 2);
        const float f = exp2f((src[0] - m) * scale_log2e);
        l += src[1] * f;
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] += src[2 + d0 + j] * f;
      }
    }
    const size_t item = (size_t)seq * n_heads + kv_head * G + h;
    if (n_splits == 1) {
      const float inv = l > 0.f ? 1.f / l : 0.f;  // no key at all (kv_len = 0): output 0
      u32x4 ov;
#pragma unroll
      for (int j = 0; j < 4; ++j) ov[j] = pack_bf16(a[2 * j] * inv, a[2 * j + 1] * inv);
      st16(o + item * HD + d0, ov);
    } else {
      float* dst = partial + (item * n_splits + split) * (HD + 2);
      if ((tid & 15) == 0) {
        dst[0] = m;
        dst[1] = l;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) dst[2 + d0 + j] = a[j];
    }
  }
}

// The grouped-query kernel: head size 128, 2..16 query heads per key/value head.
static bool gqa_kernel_serves(int n_heads, int n_kv_heads, int head_dim) {
  if (n_kv_heads <= 0 || n_heads % n_kv_heads != 0) return false;
  const int G = n_heads / n_kv_heads;
  return head_dim == kGqaHD && G >= 2 && G <= 16;
}

// Enough workgroups to cover the chip about twice, but never less than 8 pages per split.  A workgroup
// serves one (sequence, head), or one (sequence, key/value head) in the grouped-query kernel.
int decode_attention_splits(int B, int n_heads, int n_kv_heads, int head_dim, int max_kv_len) {
  const int pages = (max_kv_len + kDecPage - 1) / kDecPage;
  const long items = (long)B * (gqa_kernel_serves(n_heads, n_kv_heads, head_dim) ? n_kv_heads : n_heads);
  int splits = (int)((2 * 256 + items - 1) / items);
  const int max_splits = (pages + 2 * kDecWaves - 1) / (2 * kDecWaves);
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  return splits;
}

size_t decode_attention_workspace_bytes(int B, int n_heads, int n_kv_heads, int head_dim, int max_kv_len) {
  const int splits = decode_attention_splits(B, n_heads, n_kv_heads, head_dim, max_kv_len);
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
  const int splits = decode_attention_splits(B, n_heads, n_kv_heads, head_dim, max_kv_len);
  const int pages = (max_kv_len + kDecPage - 1) / kDecPage;
  const int pps = (pages + splits - 1) / splits;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
  const dim3 grid(n_heads, B, splits);
  if (gqa_kernel_serves(n_heads, n_kv_heads, head_dim)) {
    hipLaunchKernelGGL(decode_attention_gqa_kernel, dim3(n_kv_heads, B, splits), dim3(kDecThreads), 0, stream,
                       (const uint16_t*)q, q_stride, kv_lens, kv_len_add, block_tables, max_blocks,
                       (const uint16_t*)k_cache, (const uint16_t*)v_cache, n_heads, n_kv_heads, pps, scale_log2e,
                       (uint16_t*)o, (float*)workspace);
    if (splits > 1)
      hipLaunchKernelGGL(decode_combine_kernel<128>, dim3(B * n_heads), dim3(128), 0, stream,
                         (const float*)workspace, splits, scale_log2e, (uint16_t*)o);
  } else if (head_dim == 128) {
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
