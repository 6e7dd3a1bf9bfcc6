// Decode-phase GEMM: Y[M,N] = act(X[M,K] W[N,K]^T + bias) + residual for a handful of rows
// (the library routes M <= 128 here; the kernels accept up to 256).
// The weights (N*K*2 bytes) are read once from HBM and dominate the traffic
// (App. A.3: 4h^2 + 2hm elements per layer), so the kernels are organised
// around streaming W at HBM rate while the matrix cores do the M x ... work.
//
// Two streaming kernels live here, plus the second passes of split-K:
//   * wring_gemm_kernel  - wave-private rings, no split of K over workgroups, no second launch;
//     taken for M <= 64 when N alone yields enough workgroups (described at the kernel).
//   * skinny_gemm_kernel - one ring per workgroup, K split over workgroups; everything else.
//   * skinny_reduce*_kernel - add the split partials in a fixed order and apply the epilogue,
//     optionally fused with the LayerNorm that follows or with the append to the paged KV cache;
//     also used by the tile GEMM when it splits K.
//
// What bounds the ring kernel on this chip is the number of bytes a CU can pull through
// its vector L1 per unit time, and the activation slabs count against that
// budget although they come from L2.  A workgroup therefore covers BN = 64,
// 128 or 256 weight rows (the X slab is fetched once per BN columns), and the
// K axis is split over workgroups until the chip is full; the launcher picks
// BN and the split count that minimise weight + activation + partial-sum
// bytes.
//
// grid = (N/BN, KSPLIT).  Workgroup = 8 waves: wave w owns the column tiles
// (16 weight rows each) of column group w & 3 and, of every 128-wide k slab,
// the two 32-wide MFMA k-steps 2*(w>>2), 2*(w>>2)+1; the two k-halves are
// added through LDS at the end.  Both operands go global -> LDS directly (no
// registers, no ds_write) into a ring of S stages; a wave-level load fetches
// 4 rows x 256 contiguous bytes.  The tile is computed transposed (weights
// as MFMA row operand), so a lane ends up with 4 consecutive output columns
// of one row.  With KSPLIT > 1 each split writes fp32 partial sums and a
// second kernel adds them in a fixed order and applies the epilogue.
#include "common.h"
#include "kernels.h"

namespace ds {

// Cache policy operand of the direct-to-LDS weight loads: 2 = non-temporal.  A weight byte is used once per
// launch, so it is not worth a line in L2 or the last-level cache (measured: 42.4 -> 41.3 us per decode GEMM
// at OPT-13B, batch 64); the activation slabs, re-read by every workgroup, keep the default policy.
constexpr int kWeightAux = 2;
constexpr int kSkThreads = 512;
constexpr int kSkWaves = kSkThreads / 64;
constexpr int kSkKS = 128;  // k elements per slab

struct SkinnyParams {
  const uint16_t* X;
  const uint16_t* W;
  const uint16_t* bias;
  const uint16_t* residual;
  uint16_t* out[3];
  int seg_cols, seg_cols_kv;  // widths of the first and of the other two output segments
  int M, N, K;
  int relu;
  float* partial;  // [KSPLIT][M][N] fp32 when gridDim.y > 1
  // Greedy-choice mode (unsplit launches only): nothing is written to `out`; per row the largest
  // accumulator of this workgroup's columns and its column go to amax_val / amax_idx [gridDim.x][M].
  float* amax_val = nullptr;
  int32_t* amax_idx = nullptr;
  // Wave-private-ring kernel only: with kv_k_cache set (decode QKV projection, N = (n + 2 n_kv) s) the K and V
  // parts of row m go to slot kv_ctx_lens[m] of the paged cache [num_blocks, n_kv, 16, s] instead of `out`.
  const int32_t* kv_ctx_lens = nullptr;
  const int32_t* kv_block_tables = nullptr;
  int kv_max_blocks = 0;
  uint16_t* kv_k_cache = nullptr;
  uint16_t* kv_v_cache = nullptr;
  int kv_n_heads = 0, kv_n_kv_heads = 0, kv_head_dim = 0;
};

template <int VM>
__device__ __forceinline__ void sk_wait_vmcnt() {
  // s_waitcnt with only vmcnt set: vmcnt[3:0] | expcnt=7 | lgkmcnt=15 | vmcnt[5:4] in bits 15:14
  __builtin_amdgcn_s_waitcnt((VM & 0xf) | (0x7 << 4) | (0xf << 8) | ((VM >> 4) << 14));
}

// MT = activation row tiles of 16 (4, 8, 16); NTW = column tiles per wave (1, 2, 4: BN = 64 * NTW);
// S = LDS stages (prefetch distance D = S - 1).
//
// Stage layout: [MP rows of X | BN rows of W], every row 128 k-elements = 256 B = 16 chunks of
// 16 B, unpadded; chunk c of row r sits at position c ^ (r & 15), so the 16 consecutive rows a
// fragment read touches fall into 16 different bank groups.  The swizzle is applied on the global
// side: lane l of a wave-level load fetches row 4g + l/16, chunk (l%16) ^ (row & 15).
template <int MT, int NTW, int S>
__global__ __launch_bounds__(kSkThreads) void skinny_gemm_kernel(const SkinnyParams p) {
  constexpr int MP = MT * 16;   // padded activation rows held in LDS
  constexpr int BN = 64 * NTW;  // weight rows per workgroup
  constexpr int D = S - 1;      // slabs in flight ahead of the one being multiplied
  constexpr int STAGE_ELEMS = (MP + BN) * kSkKS;
  constexpr int GROUPS = (MP + BN) / 4;  // wave-level loads (4 rows each) per slab
  static_assert(GROUPS % kSkWaves == 0, "every wave issues the same number of loads");
  constexpr int G = GROUPS / kSkWaves;  // loads per wave per slab
  static_assert(D >= 1 && (D - 1) * G < 64, "vmcnt range");
  extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];  // [S][MP + BN][128]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int ng = wave & 3, kh = wave >> 2;  // column group, k half
  const int n0 = blockIdx.x * BN;
  const int split = blockIdx.y;
  const int n_splits = gridDim.y;
  // The K axis is dealt to the splits slab by slab (split s takes slabs s, s + KSPLIT, ...).
  const int slabs_total = p.K / kSkKS;
  const int ns = (slabs_total - split + n_splits - 1) / n_splits;  // >= 1: n_splits <= slabs_total
  const int K = p.K;

  // load j of this wave is row group g = j*8 + wave of the stage (4 rows): X rows first, then W rows
  const int lr = lane >> 4;
  const uint16_t* src[G];
#pragma unroll
  for (int j = 0; j < G; ++j) {
    const int r = 4 * (j * kSkWaves + wave) + lr;  // stage row
    const int sw = ((lane & 15) ^ (r & 15)) * 8;
    if (r < MP) src[j] = p.X + (size_t)min(r, p.M - 1) * K + (size_t)split * kSkKS + sw;
    else src[j] = p.W + (size_t)min(n0 + r - MP, p.N - 1) * K + (size_t)split * kSkKS + sw;
  }
  // requests slab i (clamped to the last real slab: a harmless re-load) into stage `st`
  auto request = [&](int i, int st) {
    const int ofs = min(i, ns - 1) * n_splits * kSkKS;
    uint16_t* dst = lds + st * STAGE_ELEMS + wave_s * 512;  // one wave-load = 4 rows = 1 KB = 512 elements
#pragma unroll
    for (int j = 0; j < G; ++j) {
      if (j < MP / (4 * kSkWaves))  // activation rows
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + ofs),
                                         (__attribute__((address_space(3))) void*)(dst + j * kSkWaves * 512), 16,
                                         0, 0);
      else
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + ofs),
                                         (__attribute__((address_space(3))) void*)(dst + j * kSkWaves * 512), 16,
                                         0, kWeightAux);
    }
  };

  floatx4 acc[NTW][MT];
#pragma unroll
  for (int a = 0; a < NTW; ++a)
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[a][t] = floatx4{0.f, 0.f, 0.f, 0.f};

  // fragment read offsets of this wave's two k-steps: lane (row = lane%16, kq = lane/16) reads
  // chunk 4*step + kq of its row
  int fo[2];
#pragma unroll
  for (int s = 0; s < 2; ++s)
    fo[s] = (lane & 15) * kSkKS + (((4 * (2 * kh + s) + (lane >> 4)) ^ (lane & 15)) * 8);
  const int wfrag0 = (MP + ng * NTW * 16) * kSkKS;

#pragma unroll
  for (int d = 0; d < D; ++d) request(d, d);

  int st = 0;      // stage of slab i
  int st_req = D;  // stage slab i+D goes to (= the stage slab i-1 used)
  for (int i = 0; i < ns; ++i) {
    sk_wait_vmcnt<(D - 1) * G>();  // this wave's part of slab i has landed
    __syncthreads();               // slab i visible to all waves; everyone is done with slab i-1
    request(i + D, st_req);
    const uint16_t* sb = lds + st * STAGE_ELEMS;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      u32x4 xf[MT];
#pragma unroll
      for (int t = 0; t < MT; ++t) xf[t] = *reinterpret_cast<const u32x4*>(sb + t * 16 * kSkKS + fo[s]);
#pragma unroll
      for (int a = 0; a < NTW; ++a) {
        const u32x4 wf = *reinterpret_cast<const u32x4*>(sb + wfrag0 + a * 16 * kSkKS + fo[s]);
#pragma unroll
        for (int t = 0; t < MT; ++t)
          acc[a][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf),
                                                              __builtin_bit_cast(bf16x8, xf[t]), acc[a][t], 0, 0, 0);
      }
    }
    st_req = st;
    st = (st + 1 == S) ? 0 : st + 1;
  }
  sk_wait_vmcnt<0>();  // no global->LDS write of this workgroup may still be in flight ...
  __syncthreads();     // ... and nobody reads the stages any more: reuse them to add the two k-halves
  {
    floatx4* red = reinterpret_cast<floatx4*>(lds);  // [4 column groups][NTW][MT][64 lanes]
    if (kh == 1) {
#pragma unroll
      for (int a = 0; a < NTW; ++a)
#pragma unroll
        for (int t = 0; t < MT; ++t) red[((ng * NTW + a) * MT + t) * 64 + lane] = acc[a][t];
    }
    __syncthreads();
    if (kh == 1) return;
#pragma unroll
    for (int a = 0; a < NTW; ++a)
#pragma unroll
      for (int t = 0; t < MT; ++t) acc[a][t] += red[((ng * NTW + a) * MT + t) * 64 + lane];
  }

  // acc[a][t][r]: row m = 16t + lane%16, column n = n0 + 16*(ng*NTW + a) + 4*(lane/16) + r
  if (p.amax_val) {
    // candidates of this lane per row tile, then across the 4 lanes that share a row (lane/16), then
    // across the 4 column-group waves through LDS (behind the k-half buffer, which may still be read)
    constexpr int RED_FLOATS = 4 * NTW * MT * 64 * 4;
    float* cv = reinterpret_cast<float*>(lds) + RED_FLOATS;  // [4 waves][MT][16]
    int32_t* ci = reinterpret_cast<int32_t*>(cv + 4 * MT * 16);
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      float bv = -INFINITY;
      int bi = 0x7fffffff;
#pragma unroll
      for (int a = 0; a < NTW; ++a)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int n = n0 + (ng * NTW + a) * 16 + (lane >> 4) * 4 + r;
          const float v = acc[a][t][r];
          if (n < p.N && (v > bv || (v == bv && n < bi))) {
            bv = v;
            bi = n;
          }
        }
#pragma unroll
      for (int off = 16; off <= 32; off <<= 1) {
        const float ov = __shfl_xor(bv, off, 64);
        const int oi = __shfl_xor(bi, off, 64);
        if (ov > bv || (ov == bv && oi < bi)) {
          bv = ov;
          bi = oi;
        }
      }
      if (lane < 16) {
        cv[(ng * MT + t) * 16 + lane] = bv;
        ci[(ng * MT + t) * 16 + lane] = bi;
      }
    }
    __syncthreads();  // the four remaining waves (the k-half-1 waves have left)
    if (ng == 0) {
      for (int e = lane; e < MT * 16; e += 64) {  // e = 16 t + row-in-tile = row m
        float bv = cv[e];
        int bi = ci[e];
#pragma unroll
        for (int g = 1; g < 4; ++g) {
          const float ov = cv[g * MT * 16 + e];
          const int oi = ci[g * MT * 16 + e];
          if (ov > bv || (ov == bv && oi < bi)) {
            bv = ov;
            bi = oi;
          }
        }
        if (e < p.M) {
          p.amax_val[(size_t)blockIdx.x * p.M + e] = bv;
          p.amax_idx[(size_t)blockIdx.x * p.M + e] = bi;
        }
      }
    }
    return;
  }
#pragma unroll
  for (int a = 0; a < NTW; ++a) {
    const int n = n0 + (ng * NTW + a) * 16 + (lane >> 4) * 4;
    if (n >= p.N) continue;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int m = t * 16 + (lane & 15);
      if (m >= p.M) continue;
      if (n_splits > 1) {
        *reinterpret_cast<floatx4*>(p.partial + ((size_t)split * p.M + m) * p.N + n) = acc[a][t];
        continue;
      }
      float v0 = acc[a][t][0], v1 = acc[a][t][1], v2 = acc[a][t][2], v3 = acc[a][t][3];
      if (p.bias) {
        const u32x2 bb = *reinterpret_cast<const u32x2*>(p.bias + n);
        v0 += bf16_lo(bb[0]); v1 += bf16_hi(bb[0]);
        v2 += bf16_lo(bb[1]); v3 += bf16_hi(bb[1]);
      }
      if (p.relu) {
        v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f);
        v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f);
      }
      if (p.residual) {
        const u32x2 rr = *reinterpret_cast<const u32x2*>(p.residual + (size_t)m * p.N + n);
        v0 += bf16_lo(rr[0]); v1 += bf16_hi(rr[0]);
        v2 += bf16_lo(rr[1]); v3 += bf16_hi(rr[1]);
      }
      const int seg = (n >= p.seg_cols) + (n >= p.seg_cols + p.seg_cols_kv);
      const int ld = seg == 0 ? p.seg_cols : p.seg_cols_kv;
      const int first = seg == 0 ? 0 : p.seg_cols + (seg - 1) * p.seg_cols_kv;
      u32x2 ov;
      ov[0] = pack_bf16(v0, v1);
      ov[1] = pack_bf16(v2, v3);
      *reinterpret_cast<u32x2*>(p.out[seg] + (size_t)m * ld + (n - first)) = ov;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Wave-private rings (up to 64 rows, wide N): the shape for which the ring kernel above needs
// split-K only to find 256 workgroups, and then pays for it twice (≈ 5 us of partial-sum stores at
// the end of every workgroup at once, ≈ 5 us for the reduce launch).  Measured on this chip: what a
// streaming kernel needs is not many bytes in flight per CU but several streams per CU that do not
// stall together - two independent 16 KB streams per CU reach 5.7 TB/s, one 64 KB stream 5.3.
//
// So: a workgroup (4 waves; 3 for batches above 64 rows) owns 64 or 80 output columns over the whole K; its waves split K between them
// 64-wide slab by slab (wave w takes slabs w, w+4, ...) and each wave runs its OWN two- or three-stage
// direct-to-LDS ring [16, 32 or 64 activation rows | 64 or 80 weight rows] x 128 bytes, waiting on nothing but its
// own loads - no barrier in the loop, four desynchronised streams per CU.  The four waves' 64 x 64
// fp32 tiles are added through LDS at the end (fixed order) and wave w finishes column tile w.
// grid = N / 64 workgroups, no partial sums in global memory, no second launch.
// ---------------------------------------------------------------------------------------------
constexpr int kWrKS = 64;  // k elements per slab

// NT = weight row tiles of 16 per workgroup (4 or 5: 64 or 80 output columns, whichever tiles N into
// fewer rounds of 256 workgroups); MT = activation row tiles of 16 (1, 2 or 4: batches of up to 16, 32 or
// 64 sequences - a small batch does not pay for 64 activation rows per slab: worth 2 us of a 158 us step at
// OPT-13B, the rest of such a step is weight bytes and per-launch ramps); S = stages of a wave's ring (the
// smaller stages of small batches leave room for a third: two slabs in flight per wave); NW = waves per
// workgroup (4; 3 for batches of 65..128 sequences, whose stages of 128 activation rows fit the LDS three times
// two, not four times two).
template <int NT, int MT, int S, int NW>
__global__ __launch_bounds__(64 * NW) void wring_gemm_kernel(const SkinnyParams p) {
  constexpr int kWrBN = 16 * NT, kWrBM = 16 * MT;
  constexpr int kWrStageElems = (kWrBM + kWrBN) * kWrKS;  // [BM X rows | BN W rows] x 64 k
  constexpr int kWrLoads = (kWrBM + kWrBN) / 8;           // wave-level loads (8 rows x 128 B) per slab
  static_assert((S - 1) * kWrLoads < 64, "vmcnt range");
  extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n0 = blockIdx.x * kWrBN;
  const int K = p.K;
  const int slabs_total = K / kWrKS;
  const int ns = (slabs_total - wave + NW - 1) / NW;  // this wave's slabs: wave, wave + NW, ...  (>= 1: K >= 256)

  // load j of a slab covers stage rows 8j .. 8j+7 (rows 0..BM-1 = X, then W); lane: row 8j + lane/8,
  // 16-byte chunk (lane%8) ^ ((row >> 1) & 7) - the swizzle that makes the fragment reads conflict-free
  const uint16_t* src[kWrLoads];
#pragma unroll
  for (int j = 0; j < kWrLoads; ++j) {
    const int r = 8 * j + (lane >> 3);
    const int sw = ((lane & 7) ^ ((r >> 1) & 7)) * 8;
    if (r < kWrBM) src[j] = p.X + (size_t)min(r, p.M - 1) * K + (size_t)wave * kWrKS + sw;
    else src[j] = p.W + (size_t)min(n0 + r - kWrBM, p.N - 1) * K + (size_t)wave * kWrKS + sw;
  }
  uint16_t* ring = lds + wave * S * kWrStageElems;
  auto request = [&](int i, int st) {  // this wave's slab i (clamped: a harmless re-load) into its stage st
    const int ofs = min(i, ns - 1) * NW * kWrKS;
    uint16_t* dst = ring + st * kWrStageElems;
#pragma unroll
    for (int j = 0; j < kWrLoads; ++j) {
      if (j < kWrBM / 8)  // activation rows
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + ofs),
                                         (__attribute__((address_space(3))) void*)(dst + j * 512), 16, 0, 0);
      else
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + ofs),
                                         (__attribute__((address_space(3))) void*)(dst + j * 512), 16, 0, kWeightAux);
    }
  };

  floatx4 acc[NT][MT];  // [weight row tile a][activation row tile t]
#pragma unroll
  for (int a = 0; a < NT; ++a)
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[a][t] = floatx4{0.f, 0.f, 0.f, 0.f};
  // fragment of k-step s (32 k): lane (row r = lane%16 of a 16-row tile, quarter q = lane/16) reads chunk 4s+q
  int fo[2];
#pragma unroll
  for (int s2 = 0; s2 < 2; ++s2)
    fo[s2] = (lane & 15) * kWrKS + (((4 * s2 + (lane >> 4)) ^ (((lane & 15) >> 1) & 7)) * 8);

#pragma unroll
  for (int i = 0; i < S - 1; ++i) request(i, i);
  int st = 0, st_in = S - 1;  // stage read in this iteration; stage the newest request goes into
  for (int i = 0; i < ns; ++i) {
    request(i + S - 1, st_in);            // that stage was last read in iteration i-1
    sk_wait_vmcnt<(S - 1) * kWrLoads>();  // slab i has landed (the S-1 younger ones may still fly)
    const uint16_t* sb = ring + st * kWrStageElems;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      u32x4 xf[MT];
#pragma unroll
      for (int t = 0; t < MT; ++t) xf[t] = *reinterpret_cast<const u32x4*>(sb + t * 16 * kWrKS + fo[s2]);
#pragma unroll
      for (int a = 0; a < NT; ++a) {
        const u32x4 wf = *reinterpret_cast<const u32x4*>(sb + (kWrBM + a * 16) * kWrKS + fo[s2]);
#pragma unroll
        for (int t = 0; t < MT; ++t)
          acc[a][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf),
                                                              __builtin_bit_cast(bf16x8, xf[t]), acc[a][t], 0, 0, 0);
      }
    }
    st = st + 1 == S ? 0 : st + 1;
    st_in = st_in + 1 == S ? 0 : st_in + 1;
  }
  sk_wait_vmcnt<0>();  // the clamped re-load of the last iteration must not land in the reduction area
  __syncthreads();     // every wave is done with its ring: reuse the LDS to add the four waves' tiles
  {
    floatx4* red = reinterpret_cast<floatx4*>(lds);  // [wave][a][t][64 lanes]
#pragma unroll
    for (int a = 0; a < NT; ++a)
#pragma unroll
      for (int t = 0; t < MT; ++t) red[((wave * NT + a) * MT + t) * 64 + lane] = acc[a][t];
    __syncthreads();
  }
  // wave w finishes weight row tiles a = w (and w + 4): the four waves' tiles are added in wave order.
  // Lane: row m = 16t + lane%16, columns n = n0 + 16a + 4*(lane/16) + 0..3.
  const floatx4* red = reinterpret_cast<const floatx4*>(lds);
  for (int a = wave; a < NT; a += NW) {
    const int n = n0 + 16 * a + (lane >> 4) * 4;
    if (n >= p.N) continue;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int m = t * 16 + (lane & 15);
      if (m >= p.M) continue;
      floatx4 v = red[((0 * NT + a) * MT + t) * 64 + lane];
#pragma unroll
      for (int w2 = 1; w2 < NW; ++w2) v += red[((w2 * NT + a) * MT + t) * 64 + lane];
      float v0 = v[0], v1 = v[1], v2 = v[2], v3 = v[3];
      if (p.bias) {
        const u32x2 bb = *reinterpret_cast<const u32x2*>(p.bias + n);
        v0 += bf16_lo(bb[0]); v1 += bf16_hi(bb[0]);
        v2 += bf16_lo(bb[1]); v3 += bf16_hi(bb[1]);
      }
      if (p.relu) {
        v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f);
        v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f);
      }
      if (p.residual) {
        const u32x2 rr = *reinterpret_cast<const u32x2*>(p.residual + (size_t)m * p.N + n);
        v0 += bf16_lo(rr[0]); v1 += bf16_hi(rr[0]);
        v2 += bf16_lo(rr[1]); v3 += bf16_hi(rr[1]);
      }
      u32x2 ov;
      ov[0] = pack_bf16(v0, v1);
      ov[1] = pack_bf16(v2, v3);
      const int hq = p.kv_n_heads * p.kv_head_dim, hkv = p.kv_n_kv_heads * p.kv_head_dim;
      if (p.kv_k_cache && n >= hq) {  // decode QKV projection: this step's K / V row goes straight into its page
        const int which = n >= hq + hkv;
        const int col = n - hq - which * hkv;
        const int head = col / p.kv_head_dim, d = col - head * p.kv_head_dim;
        const int pos = p.kv_ctx_lens[m];
        const int blk = p.kv_block_tables[(size_t)m * p.kv_max_blocks + pos / 16];
        uint16_t* dst = (which ? p.kv_v_cache : p.kv_k_cache) +
                        (((size_t)blk * p.kv_n_kv_heads + head) * 16 + (pos % 16)) * p.kv_head_dim + d;
        *reinterpret_cast<u32x2*>(dst) = ov;
        continue;
      }
      const int seg = (n >= p.seg_cols) + (n >= p.seg_cols + p.seg_cols_kv);
      const int ld = seg == 0 ? p.seg_cols : p.seg_cols_kv;
      const int first = seg == 0 ? 0 : p.seg_cols + (seg - 1) * p.seg_cols_kv;
      *reinterpret_cast<u32x2*>(p.out[seg] + (size_t)m * ld + (n - first)) = ov;
    }
  }
}

// Sum of the split partials of 8 consecutive columns of row m, added in split order; the loads of four
// splits are issued together (the reduce passes are latency-bound).
__device__ __forceinline__ void sum_partials8(const SkinnyParams& p, int n_splits, int m, int n, float v[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = 0.f;
  for (int s0 = 0; s0 < n_splits; s0 += 4) {
    floatx4 a[4], b[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float* src = p.partial + ((size_t)min(s0 + u, n_splits - 1) * p.M + m) * p.N + n;
      a[u] = *reinterpret_cast<const floatx4*>(src);
      b[u] = *reinterpret_cast<const floatx4*>(src + 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (s0 + u < n_splits) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[j] += a[u][j];
          v[4 + j] += b[u][j];
        }
      }
    }
  }
}

// Sum the split partials in split order, then bias / ReLU / residual, 8 columns per thread.
__global__ __launch_bounds__(256) void skinny_reduce_kernel(const SkinnyParams p, int n_splits) {
  const int chunks_per_row = p.N >> 3;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)p.M * chunks_per_row) return;
  const int m = (int)(idx / chunks_per_row);
  const int n = (int)(idx % chunks_per_row) * 8;
  float v[8];
  sum_partials8(p, n_splits, m, n, v);
  if (p.bias) {
    const u32x4 bb = ld16(p.bias + n);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[2 * j] += bf16_lo(bb[j]);
      v[2 * j + 1] += bf16_hi(bb[j]);
    }
  }
  if (p.relu) {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = fmaxf(v[j], 0.f);
  }
  if (p.residual) {
    const u32x4 rr = ld16(p.residual + (size_t)m * p.N + n);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[2 * j] += bf16_lo(rr[j]);
      v[2 * j + 1] += bf16_hi(rr[j]);
    }
  }
  const int seg = (n >= p.seg_cols) + (n >= p.seg_cols + p.seg_cols_kv);
  const int ld = seg == 0 ? p.seg_cols : p.seg_cols_kv;
  const int first = seg == 0 ? 0 : p.seg_cols + (seg - 1) * p.seg_cols_kv;
  u32x4 ov;
#pragma unroll
  for (int j = 0; j < 4; ++j) ov[j] = pack_bf16(v[2 * j], v[2 * j + 1]);
  st16(p.out[seg] + (size_t)m * ld + (n - first), ov);
}

// The same reduction, one workgroup per output row, followed by LayerNorm of that row: writes
// out[0][m,:] = act(sum + bias) + residual (bf16) and ln_out[m,:] = LN(out[m,:]) (statistics in
// fp32 over the bf16-rounded row, exactly what the stand-alone LayerNorm kernel would see).
// 1024 threads per row so that a 5120-wide row is one 8-column piece per thread and all partial loads of a
// row are in flight together (the kernel is pure latency: 64 rows, a few hundred KB each).
constexpr int kRedLnThreads = 1024;
constexpr int kRedLnMaxChunks = 2;  // 2 pieces x 8 columns x 1024 threads = 16384 columns
template <int NCH>
__global__ __launch_bounds__(kRedLnThreads) void skinny_reduce_ln_kernel(const SkinnyParams p, int n_splits,
                                                                         const uint16_t* __restrict__ gamma,
                                                                         const uint16_t* __restrict__ beta, float eps,
                                                                         uint16_t* __restrict__ ln_out) {
  __shared__ float red[kRedLnThreads / 64];
  const int m = blockIdx.x;
  const int nchunk = p.N >> 3;
  float vals[NCH][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = threadIdx.x + i * kRedLnThreads;
    if (c < nchunk) {
      const int n = c * 8;
      float v[8];
      sum_partials8(p, n_splits, m, n, v);
      if (p.bias) {
        const u32x4 bb = ld16(p.bias + n);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[2 * j] += bf16_lo(bb[j]);
          v[2 * j + 1] += bf16_hi(bb[j]);
        }
      }
      if (p.relu) {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = fmaxf(v[j], 0.f);
      }
      if (p.residual) {
        const u32x4 rr = ld16(p.residual + (size_t)m * p.N + n);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[2 * j] += bf16_lo(rr[j]);
          v[2 * j + 1] += bf16_hi(rr[j]);
        }
      }
      u32x4 ov;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        ov[j] = pack_bf16(v[2 * j], v[2 * j + 1]);
        vals[i][2 * j] = bf16_lo(ov[j]);
        vals[i][2 * j + 1] = bf16_hi(ov[j]);
        sum += vals[i][2 * j] + vals[i][2 * j + 1];
      }
      st16(p.out[0] + (size_t)m * p.N + n, ov);
    }
  }
  auto block_sum = [&](float v) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kRedLnThreads / 64; ++w) t += red[w];
    return t;
  };
  const float mean = block_sum(sum) / (float)p.N;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = threadIdx.x + i * kRedLnThreads;
    if (c < nchunk) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float d = vals[i][j] - mean;
        sq += d * d;
      }
    }
  }
  const float rstd = rsqrtf(block_sum(sq) / (float)p.N + eps);
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = threadIdx.x + i * kRedLnThreads;
    if (c < nchunk) {
      const u32x4 g = ld16(gamma + c * 8);
      const u32x4 b = ld16(beta + c * 8);
      u32x4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float lo = (vals[i][2 * j] - mean) * rstd * bf16_lo(g[j]) + bf16_lo(b[j]);
        const float hi = (vals[i][2 * j + 1] - mean) * rstd * bf16_hi(g[j]) + bf16_hi(b[j]);
        o[j] = pack_bf16(lo, hi);
      }
      st16(ln_out + (size_t)m * p.N + c * 8, o);
    }
  }
}

// The same reduction for the decode QKV projection (N = (n + 2 n_kv) s, one output buffer with row stride N):
// the Q part is written to out[0]; the K and V parts are this step's new cache rows and go to
// slot ctx_lens[m] of the paged cache [num_blocks, n_kv, 16, s].
__global__ __launch_bounds__(256) void skinny_reduce_kv_kernel(const SkinnyParams p, int n_splits,
                                                               const int32_t* __restrict__ ctx_lens,
                                                               const int32_t* __restrict__ block_tables,
                                                               int max_blocks, uint16_t* __restrict__ k_cache,
                                                               uint16_t* __restrict__ v_cache, int n_heads,
                                                               int n_kv_heads, int head_dim) {
  const int chunks_per_row = p.N >> 3;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)p.M * chunks_per_row) return;
  const int m = (int)(idx / chunks_per_row);
  const int n = (int)(idx % chunks_per_row) * 8;
  float v[8];
  sum_partials8(p, n_splits, m, n, v);
  if (p.bias) {
    const u32x4 bb = ld16(p.bias + n);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[2 * j] += bf16_lo(bb[j]);
      v[2 * j + 1] += bf16_hi(bb[j]);
    }
  }
  u32x4 ov;
#pragma unroll
  for (int j = 0; j < 4; ++j) ov[j] = pack_bf16(v[2 * j], v[2 * j + 1]);
  const int h = n_heads * head_dim, hkv = n_kv_heads * head_dim;
  if (n < h) {
    st16(p.out[0] + (size_t)m * p.N + n, ov);
    return;
  }
  const int which = n >= h + hkv;
  const int col = n - h - which * hkv;
  const int head = col / head_dim, d = col - head * head_dim;
  const int pos = ctx_lens[m];
  const int blk = block_tables[(size_t)m * max_blocks + pos / 16];
  uint16_t* dst = (which ? v_cache : k_cache) + (((size_t)blk * n_kv_heads + head) * 16 + (pos % 16)) * head_dim + d;
  st16(dst, ov);
}

DS_SWITCH(g_skinny_force_ntw, 0);  // 0 = byte model
DS_SWITCH(g_skinny_force_splits, 0);

struct SkinnyPlan {
  int ntw;     // column tiles per wave: BN = 64 * ntw
  int splits;  // K splits over workgroups
};

// Measured on MI355X: a CU sustains about one workgroup's worth of streaming whatever the LDS would
// allow, and a second round of workgroups costs a full round.  So a plan must fit one round
// (<= 256 workgroups) and should fill it; among such plans take the fewest bytes through the CUs' L1:
//   weights + (N/BN) * X (each column block re-reads the activations) + partial sums written and
//   read back.
static SkinnyPlan skinny_plan(int M, int N, int K, bool allow_split = true, double* cost_out = nullptr) {
  const int slabs = K / kSkKS;
  const int mp = M <= 64 ? 64 : (M <= 128 ? 128 : 256);
  SkinnyPlan best{1, 1};
  double best_cost = 1e300;
  for (int ntw = 1; ntw <= 4; ntw *= 2) {
    if (g_skinny_force_ntw > 0 && ntw != g_skinny_force_ntw) continue;
    const int bn = 64 * ntw;
    if (mp == 256 && ntw > 1) continue;  // (256 + 128) * 256 B * 2 stages does not fit the LDS
    if (mp == 128 && ntw > 2) continue;
    const int wgs_n = (N + bn - 1) / bn;
    for (int splits = 1; splits <= slabs && splits <= 64; ++splits) {
      if (!allow_split && splits > 1) break;
      if (allow_split && g_skinny_force_splits > 0 && splits != g_skinny_force_splits) continue;
      const double wgs = (double)wgs_n * splits;
      const bool forced = g_skinny_force_splits > 0;
      if (wgs > 256.0 && splits > 1 && !forced) break;        // never split into a second round
      const double rounds = wgs <= 256.0 ? 1.0 : ceil(wgs / 256.0);  // unsplit but larger than the chip: whole rounds
      const double fill = wgs >= 256.0 ? 1.0 : 256.0 / wgs;    // idle CUs stretch the time
      // partial sums are charged four times their bytes: they are stored by every workgroup at once at
      // the end of the launch and read back by a second, latency-bound launch (measured: 6 splits of
      // 128 columns beat 12 splits of 256 on the FFN-out shape although they stream more activations; charged
      // for the padded row count, since a workgroup's partial-tile epilogue costs the same at 16 rows as at 64)
      const double bytes = 2.0 * N * K + 2.0 * wgs_n * (double)mp * K +
                           (splits > 1 ? 4.0 * 2.0 * 4.0 * splits * (double)mp * N : 0.0);
      const double cost = bytes * fill * rounds;
      if (cost < best_cost) {
        best_cost = cost;
        best = SkinnyPlan{ntw, splits};
      }
    }
  }
  if (cost_out) *cost_out = best_cost + (best.splits > 1 ? 57e6 : 0.0);  // + the reduce launch (6 us of the chip)
  return best;
}

size_t skinny_workspace_bytes(int M, int N, int K) {
  if (K % kSkKS != 0 || M > 256) return 0;
  const SkinnyPlan pl = skinny_plan(M, N, K);  // (also covers the shapes the unsplit kernel takes)
  return pl.splits > 1 ? (size_t)pl.splits * M * N * sizeof(float) : 0;
}

template <int MT, int NTW, int S>
static hipError_t launch_skinny_cfg(const SkinnyParams& p, int splits, hipStream_t stream) {
  constexpr int BN = 64 * NTW;
  constexpr size_t lds_bytes = (size_t)S * (MT * 16 + BN) * kSkKS * sizeof(uint16_t);
  static_assert(lds_bytes <= 160 * 1024, "LDS");
  static_assert((size_t)4 * NTW * MT * 64 * 16 + (size_t)4 * MT * 16 * 8 <= lds_bytes,
                "k-half reduction (and the greedy-choice candidates behind it) fit the stages");
  constexpr auto kern = skinny_gemm_kernel<MT, NTW, S>;
  (void)KernelAttrReg<kern, (int)lds_bytes>::done;
  hipLaunchKernelGGL(kern, dim3((p.N + BN - 1) / BN, splits), dim3(kSkThreads), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int NT, int MT, int S, int NW>
static hipError_t launch_wring_cfg(const SkinnyParams& p, hipStream_t stream) {
  constexpr size_t lds_bytes = (size_t)NW * S * (16 * MT + 16 * NT) * kWrKS * sizeof(uint16_t);  // NW waves x S stages
  static_assert(lds_bytes <= 160 * 1024 && (size_t)NW * NT * MT * 1024 <= lds_bytes, "LDS");
  constexpr auto kern = wring_gemm_kernel<NT, MT, S, NW>;
  (void)KernelAttrReg<kern, (int)lds_bytes>::done;
  hipLaunchKernelGGL(kern, dim3((p.N + 16 * NT - 1) / (16 * NT)), dim3(64 * NW), lds_bytes, stream, p);
  return hipGetLastError();
}

// The instantiation for NT column tiles and the batch's row count.
static hipError_t launch_wring(int nt, const SkinnyParams& p, hipStream_t stream) {
  const int M = p.M;
  if (nt == 5) {
    if (M <= 16) return launch_wring_cfg<5, 1, 3, 4>(p, stream);  // 144 KB
    if (M <= 32) return launch_wring_cfg<5, 2, 2, 4>(p, stream);  // 112 KB
    if (M <= 64) return launch_wring_cfg<5, 4, 2, 4>(p, stream);  // 144 KB
    return launch_wring_cfg<5, 8, 2, 3>(p, stream);               // 156 KB
  }
  if (M <= 16) return launch_wring_cfg<4, 1, 3, 4>(p, stream);    // 120 KB
  if (M <= 32) return launch_wring_cfg<4, 2, 3, 4>(p, stream);    // 144 KB
  if (M <= 64) return launch_wring_cfg<4, 4, 2, 4>(p, stream);    // 128 KB
  return launch_wring_cfg<4, 8, 2, 3>(p, stream);                 // 144 KB
}

// Column-tile width (in 16-row tiles) for the wave-private-ring kernel, or 0 if the shape is not one it
// is good at: K a multiple of 256 and enough column tiles to occupy most of the chip without splitting K.
// Up to 64 rows it takes both widths; for 65..128 rows only the 80-column one, where a workgroup re-reads 1.6
// activation bytes per weight byte rather than 2 (measured at 128 rows: FFN-in of OPT-13B / 66B and QKV of
// OPT-175B 18-27 % faster than the split-K ring kernel, every 64-column shape equal or up to 20 % slower).
DS_SWITCH(g_skinny_wring, 1);  // 0 = never use the wave-private-ring kernel, 2 = also where it needs several rounds
static int wring_tiles(int M, int N, int K) {
  if (!g_skinny_wring || M > 128 || K < 256 || K % 256 != 0) return 0;
  const int t4 = (N + 63) / 64, t5 = (N + 79) / 80;
  const int r4 = (t4 + 255) / 256, r5 = (t5 + 255) / 256;
  const int nt = r5 < r4 ? 5 : 4;
  const int tiles = nt == 5 ? t5 : t4;
  if (M > 64 && nt != 5) return 0;
  if (tiles < 160) return 0;
  // Several rounds of workgroups: each of them streams the activation slab again beside its 64 or 80 weight
  // rows, and from 32 rows up that is as many bytes through a compute unit's load path as the weights.  The
  // split-K ring kernel with 256-column tiles reads a quarter of that and stays within one round; it wins where
  // its bytes (in skinny_plan's terms, reduce launch included) are clearly fewer.  Measured at 64 rows: FFN-in of
  // OPT-175B 245 -> 214 us, QKV of OPT-66B 107 -> 98 us; QKV of OPT-175B and FFN-in of OPT-66B (two rounds of 80
  // columns against 144 workgroups of 256) stay here, 6-9 % ahead.
  const int rounds = nt == 5 ? r5 : r4;
  if (rounds > 1 && M > 16 && g_skinny_wring != 2) {
    const double rows = M <= 32 ? 32 : (M <= 64 ? 64 : 128);
    const double wring_cost = rounds * 256.0 * (16.0 * nt + rows) * K * 2.0;
    double ring_cost;
    skinny_plan(M, N, K, true, &ring_cost);
    if (ring_cost < 0.95 * wring_cost) return 0;
  }
  return nt;
}

static hipError_t dispatch_skinny(const SkinnyParams& p, const SkinnyPlan& pl, hipStream_t stream) {
  // fewer than 64 rows run as 64 (clamped duplicates; the matrix cores are idle anyway)
  if (p.M <= 64) {
    if (pl.ntw == 4) return launch_skinny_cfg<4, 4, 2>(p, pl.splits, stream);  // 160 KB
    if (pl.ntw == 2) return launch_skinny_cfg<4, 2, 3>(p, pl.splits, stream);  // 144 KB
    return launch_skinny_cfg<4, 1, 2>(p, pl.splits, stream);                   //  64 KB
  }
  if (p.M <= 128) {
    if (pl.ntw == 2) return launch_skinny_cfg<8, 2, 2>(p, pl.splits, stream);  // 128 KB
    return launch_skinny_cfg<8, 1, 3>(p, pl.splits, stream);                   // 144 KB
  }
  return launch_skinny_cfg<16, 1, 2>(p, pl.splits, stream);                    // 160 KB
}

hipError_t launch_argmax_merge(const float* part_val, const int32_t* part_idx, int n_blocks, int M,
                               int32_t* next_token, float* best_logit, hipStream_t stream);

size_t skinny_argmax_workspace_bytes(int M, int N, int K) {
  if (K % kSkKS != 0 || M > 256 || M <= 0 || N <= 0) return 0;
  const SkinnyPlan pl = skinny_plan(M, N, K, false);
  const size_t blocks = (size_t)(N + 64 * pl.ntw - 1) / (64 * pl.ntw);
  return blocks * M * (sizeof(float) + sizeof(int32_t));
}

hipError_t launch_skinny_argmax(const void* X, const void* W, int M, int N, int K, void* workspace,
                                int32_t* next_token, float* best_logit, hipStream_t stream) {
  if (M <= 0 || M > 256 || N <= 0 || K % kSkKS != 0 || !workspace || !next_token) return hipErrorInvalidValue;
  const SkinnyPlan pl = skinny_plan(M, N, K, false);
  const int blocks = (N + 64 * pl.ntw - 1) / (64 * pl.ntw);
  SkinnyParams p;
  p.X = (const uint16_t*)X;
  p.W = (const uint16_t*)W;
  p.bias = nullptr;
  p.residual = nullptr;
  for (int i = 0; i < 3; ++i) p.out[i] = nullptr;
  p.seg_cols = N;
  p.seg_cols_kv = N;
  p.M = M; p.N = N; p.K = K;
  p.relu = 0;
  p.partial = nullptr;
  p.amax_val = (float*)workspace;
  p.amax_idx = (int32_t*)(p.amax_val + (size_t)blocks * M);
  hipError_t e = dispatch_skinny(p, pl, stream);
  if (e != hipSuccess) return e;
  return launch_argmax_merge(p.amax_val, p.amax_idx, blocks, M, next_token, best_logit, stream);
}

// Second pass of any split-K product: partial [splits][M][N] fp32 -> epilogue, optionally with the
// LayerNorm or KV-append work folded in (reported through *fused_done).
hipError_t launch_splitk_reduce(const float* partial, int splits, int M, int N, const Epilogue& ep,
                                const SkinnyFused* fused, bool* fused_done, hipStream_t stream) {
  if (fused_done) *fused_done = false;
  if (N % 8 != 0 || ep.seg_cols <= 0 || ep.seg_cols % 8 != 0 || ep.seg_cols_kv < 0 || ep.seg_cols_kv % 8 != 0)
    return hipErrorInvalidValue;
  SkinnyParams p;
  p.X = nullptr;
  p.W = nullptr;
  p.bias = (const uint16_t*)ep.bias;
  p.residual = (const uint16_t*)ep.residual;
  for (int i = 0; i < 3; ++i) p.out[i] = (uint16_t*)ep.out[i];
  p.seg_cols = ep.seg_cols;
  p.seg_cols_kv = ep.seg_cols_kv > 0 ? ep.seg_cols_kv : ep.seg_cols;
  p.M = M; p.N = N; p.K = 0;
  p.relu = ep.relu;
  p.partial = const_cast<float*>(partial);
  const long items = (long)M * (N / 8);
  const unsigned blocks = (unsigned)((items + 255) / 256);
  if (fused && fused->kind == SkinnyFused::kLayerNorm && ep.seg_cols == N &&
      N <= kRedLnThreads * 8 * kRedLnMaxChunks) {
    if (N <= kRedLnThreads * 8)
      hipLaunchKernelGGL(skinny_reduce_ln_kernel<1>, dim3(M), dim3(kRedLnThreads), 0, stream, p, splits,
                         (const uint16_t*)fused->ln_gamma, (const uint16_t*)fused->ln_beta, fused->ln_eps,
                         (uint16_t*)fused->ln_out);
    else
      hipLaunchKernelGGL(skinny_reduce_ln_kernel<2>, dim3(M), dim3(kRedLnThreads), 0, stream, p, splits,
                         (const uint16_t*)fused->ln_gamma, (const uint16_t*)fused->ln_beta, fused->ln_eps,
                         (uint16_t*)fused->ln_out);
    if (fused_done) *fused_done = true;
  } else if (fused && fused->kind == SkinnyFused::kKvAppend && ep.seg_cols == N && !ep.relu && !ep.residual &&
             N == (fused->n_heads + 2 * fused->n_kv_heads) * fused->head_dim) {
    hipLaunchKernelGGL(skinny_reduce_kv_kernel, dim3(blocks), dim3(256), 0, stream, p, splits, fused->ctx_lens,
                       fused->block_tables, fused->max_blocks, (uint16_t*)fused->k_cache,
                       (uint16_t*)fused->v_cache, fused->n_heads, fused->n_kv_heads, fused->head_dim);
    if (fused_done) *fused_done = true;
  } else {
    hipLaunchKernelGGL(skinny_reduce_kernel, dim3(blocks), dim3(256), 0, stream, p, splits);
  }
  return hipGetLastError();
}

// What launch_skinny_gemm does for a plain product of this shape: columns per workgroup and splits over K
// (1 split and 64 or 80 columns = the unsplit kernel with wave-private rings).
void skinny_describe(int M, int N, int K, int* tile_cols, int* splits) {
  if (const int nt = wring_tiles(M, N, K)) {
    *tile_cols = 16 * nt;
    *splits = 1;
    return;
  }
  const SkinnyPlan pl = skinny_plan(M, N, K);
  *tile_cols = 64 * pl.ntw;
  *splits = pl.splits;
}

hipError_t launch_skinny_gemm(const void* X, const void* W, int M, int N, int K, const Epilogue& ep,
                              void* workspace, hipStream_t stream, const SkinnyFused* fused, bool* fused_done) {
  if (fused_done) *fused_done = false;
  if (M <= 0 || N <= 0) return hipSuccess;
  if (M > 256 || K % kSkKS != 0 || N % 8 != 0 || ep.seg_cols <= 0 || ep.seg_cols % 8 != 0 || ep.seg_cols_kv < 0 ||
      ep.seg_cols_kv % 8 != 0)
    return hipErrorInvalidValue;
  if (ep.residual && ep.seg_cols != N) return hipErrorInvalidValue;
  if (ep.x_ld != 0 || ep.out_ld != 0) return hipErrorInvalidValue;  // dense rows only
  SkinnyParams p;
  p.X = (const uint16_t*)X;
  p.W = (const uint16_t*)W;
  p.bias = (const uint16_t*)ep.bias;
  p.residual = (const uint16_t*)ep.residual;
  for (int i = 0; i < 3; ++i) p.out[i] = (uint16_t*)ep.out[i];
  p.seg_cols = ep.seg_cols;
  p.seg_cols_kv = ep.seg_cols_kv > 0 ? ep.seg_cols_kv : ep.seg_cols;
  p.M = M; p.N = N; p.K = K;
  p.relu = ep.relu;
  // wide N, few rows: unsplit, wave-private rings, K/V scatter in its own epilogue
  const bool plain = !fused || fused->kind == SkinnyFused::kNone;
  const bool want_kv = fused && fused->kind == SkinnyFused::kKvAppend && ep.seg_cols == N && !ep.relu &&
                       !ep.residual && N == (fused->n_heads + 2 * fused->n_kv_heads) * fused->head_dim &&
                       fused->head_dim % 4 == 0;
  const int nt = (plain || want_kv) ? wring_tiles(M, N, K) : 0;
  if (nt > 0) {
    if (want_kv) {
      p.kv_ctx_lens = fused->ctx_lens; p.kv_block_tables = fused->block_tables; p.kv_max_blocks = fused->max_blocks;
      p.kv_k_cache = (uint16_t*)fused->k_cache; p.kv_v_cache = (uint16_t*)fused->v_cache;
      p.kv_n_heads = fused->n_heads; p.kv_n_kv_heads = fused->n_kv_heads; p.kv_head_dim = fused->head_dim;
      if (fused_done) *fused_done = true;
    }
    p.partial = nullptr;
    return launch_wring(nt, p, stream);
  }
  const SkinnyPlan pl = skinny_plan(M, N, K);
  p.partial = (float*)workspace;
  if (pl.splits > 1 && workspace == nullptr) return hipErrorInvalidValue;
  hipError_t e = dispatch_skinny(p, pl, stream);
  if (e != hipSuccess) return e;
  if (pl.splits > 1) e = launch_splitk_reduce(p.partial, pl.splits, M, N, ep, fused, fused_done, stream);
  return e;
}

}  // namespace ds
