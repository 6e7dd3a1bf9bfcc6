// bf16 GEMM on the CDNA4 matrix cores for the prefill phase:
//   Y[M,N] = act(X[M,K] W[N,K]^T + bias) + residual,  fp32 accumulate.
// Both operands are K-contiguous, so a lane's 8-element MFMA fragment is one
// 16-byte LDS read.  The kernel computes the tile transposed (weight rows as
// the MFMA row operand, activation rows as the column operand): each lane
// then owns 4 consecutive output columns of one output row, which makes the
// bias load, residual load and bf16 store 8-byte accesses.
//
// Tile BM x BN (activation rows x weight rows), BK = 64, 256 threads (4
// waves, one per SIMD), LDS double-buffered, global->register->LDS prefetch
// of tile k+1 overlapping the MFMAs of tile k.
#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kBK = 64;
constexpr int kLdsStride = kBK + 8;  // elements; 144-byte rows keep 16-byte fragment reads conflict-free
constexpr int kGemmThreads = 256;

struct GemmParams {
  const uint16_t* X;
  const uint16_t* W;
  const uint16_t* bias;
  const uint16_t* residual;
  uint16_t* out[3];
  int seg_cols;
  int M, N, K;
  int relu;
  int tiles_m, tiles_n;
};

// Workgroup ids are dealt round-robin to the 8 XCDs (each with a private L2).
// Give every XCD a contiguous range of tile ids, m-fastest, so the workgroups
// that share an L2 also share weight tiles.
__device__ __forceinline__ int xcd_remap(int pid, int total) {
  constexpr int kXcd = 8;
  const int per = total / kXcd;
  if (pid >= per * kXcd) return pid;  // tail that does not fill all XCDs
  return (pid % kXcd) * per + pid / kXcd;
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(kGemmThreads) void gemm_tn_kernel(const GemmParams p) {
  static_assert(WAVES_M * WAVES_N == 4, "4 waves");
  constexpr int WTM = BM / WAVES_M;  // activation rows per wave
  constexpr int WTN = BN / WAVES_N;  // weight rows per wave
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  constexpr int XCH = BM * (kBK / 8) / kGemmThreads;  // 16-byte chunks per thread per tile
  constexpr int WCH = BN * (kBK / 8) / kGemmThreads;
  static_assert(BM * (kBK / 8) % kGemmThreads == 0 && BN * (kBK / 8) % kGemmThreads == 0, "chunking");

  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* xs = lds;                               // [2][BM][kLdsStride]
  uint16_t* ws = lds + 2 * BM * kLdsStride;         // [2][BN][kLdsStride]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  const int tile = xcd_remap(blockIdx.x, p.tiles_m * p.tiles_n);
  const int m0 = (tile % p.tiles_m) * BM;
  const int n0 = (tile / p.tiles_m) * BN;
  const int K = p.K;

  // global chunk addresses (element offsets fit in 32 bits for every supported shape)
  uint32_t xoff[XCH], woff[WCH];
  uint32_t xlds[XCH], wlds[WCH];
#pragma unroll
  for (int i = 0; i < XCH; ++i) {
    const int c = tid + i * kGemmThreads;
    const int r = c >> 3, kc = c & 7;
    const int row = min(m0 + r, p.M - 1);
    xoff[i] = (uint32_t)row * (uint32_t)K + kc * 8;
    xlds[i] = r * kLdsStride + kc * 8;
  }
#pragma unroll
  for (int i = 0; i < WCH; ++i) {
    const int c = tid + i * kGemmThreads;
    const int r = c >> 3, kc = c & 7;
    const int row = min(n0 + r, p.N - 1);
    woff[i] = (uint32_t)row * (uint32_t)K + kc * 8;
    wlds[i] = r * kLdsStride + kc * 8;
  }

  floatx16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  u32x4 xr[XCH], wr[WCH];
  const uint16_t* Xk = p.X;
  const uint16_t* Wk = p.W;
  auto gload = [&]() {
#pragma unroll
    for (int i = 0; i < XCH; ++i) xr[i] = ld16(Xk + xoff[i]);
#pragma unroll
    for (int i = 0; i < WCH; ++i) wr[i] = ld16(Wk + woff[i]);
    Xk += kBK;
    Wk += kBK;
  };
  auto sstore = [&](int buf) {
    uint16_t* xb = xs + buf * BM * kLdsStride;
    uint16_t* wb = ws + buf * BN * kLdsStride;
#pragma unroll
    for (int i = 0; i < XCH; ++i) st16(xb + xlds[i], xr[i]);
#pragma unroll
    for (int i = 0; i < WCH; ++i) st16(wb + wlds[i], wr[i]);
  };

  const int frag_row = lane & 31;
  const int frag_k = (lane >> 5) * 8;
  const int KT = K / kBK;

  gload();
  sstore(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) gload();
    const uint16_t* xb = xs + buf * BM * kLdsStride + (wm * WTM + frag_row) * kLdsStride + frag_k;
    const uint16_t* wb = ws + buf * BN * kLdsStride + (wn * WTN + frag_row) * kLdsStride + frag_k;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 wf[TN], xf[TM];
#pragma unroll
      for (int a = 0; a < TN; ++a) wf[a] = *reinterpret_cast<const bf16x8*>(wb + a * 32 * kLdsStride + kk * 16);
#pragma unroll
      for (int b = 0; b < TM; ++b) xf[b] = *reinterpret_cast<const bf16x8*>(xb + b * 32 * kLdsStride + kk * 16);
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf[b], acc[a][b], 0, 0, 0);
    }
    if (kt + 1 < KT) sstore(buf ^ 1);
    __syncthreads();
  }

  // Epilogue.  acc[a][b][4g+i] is output row m = m0 + wm*WTM + b*32 + lane%32,
  // column n = n0 + wn*WTN + a*32 + 8g + 4*(lane/32) + i.
  const int m = m0 + wm * WTM + (lane & 31);
  const int nl = n0 + wn * WTN + (lane >> 5) * 4;
#pragma unroll
  for (int b = 0; b < TM; ++b) {
    const int row = m + b * 32;
    if (row >= p.M) continue;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = nl + a * 32 + g * 8;
        if (n >= p.N) continue;
        float v0 = acc[a][b][4 * g + 0], v1 = acc[a][b][4 * g + 1];
        float v2 = acc[a][b][4 * g + 2], v3 = acc[a][b][4 * g + 3];
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
          const u32x2 rr = *reinterpret_cast<const u32x2*>(p.residual + (size_t)row * p.N + n);
          v0 += bf16_lo(rr[0]); v1 += bf16_hi(rr[0]);
          v2 += bf16_lo(rr[1]); v3 += bf16_hi(rr[1]);
        }
        const int seg = n / p.seg_cols;
        const int col = n - seg * p.seg_cols;
        u32x2 o;
        o[0] = pack_bf16(v0, v1);
        o[1] = pack_bf16(v2, v3);
        *reinterpret_cast<u32x2*>(p.out[seg] + (size_t)row * p.seg_cols + col) = o;
      }
    }
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
static hipError_t launch_cfg(GemmParams p, hipStream_t stream) {
  p.tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N + BN - 1) / BN;
  constexpr size_t lds_bytes = 2ull * (BM + BN) * kLdsStride * sizeof(uint16_t);
  auto kern = gemm_tn_kernel<BM, BN, WAVES_M, WAVES_N>;
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(p.tiles_m * p.tiles_n), dim3(kGemmThreads), lds_bytes, stream, p);
  return hipGetLastError();
}

// Rounds of workgroups on 256 CUs (one workgroup per CU) times the padded tile
// area: the cost model used to pick a tile shape.
static double tile_cost(int M, int N, int BM, int BN) {
  const long tiles = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const long rounds = (tiles + 255) / 256;
  return (double)rounds * BM * BN;
}

hipError_t launch_gemm(const void* X, const void* W, int M, int N, int K, const Epilogue& ep,
                       hipStream_t stream) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (K % kBK != 0 || N % 8 != 0 || ep.seg_cols <= 0 || ep.seg_cols % 8 != 0) return hipErrorInvalidValue;
  GemmParams p;
  p.X = (const uint16_t*)X;
  p.W = (const uint16_t*)W;
  p.bias = (const uint16_t*)ep.bias;
  p.residual = (const uint16_t*)ep.residual;
  for (int i = 0; i < 3; ++i) p.out[i] = (uint16_t*)ep.out[i];
  p.seg_cols = ep.seg_cols;
  p.M = M; p.N = N; p.K = K;
  p.relu = ep.relu;
  p.tiles_m = p.tiles_n = 0;
  const double c_a = tile_cost(M, N, 256, 160);
  const double c_b = tile_cost(M, N, 256, 256) * 0.95;  // larger tile re-reads less per flop
  const double c_c = tile_cost(M, N, 128, 128) * 1.15;  // smaller tile pays more LDS traffic per flop
  if (c_c < c_a && c_c < c_b) return launch_cfg<128, 128, 2, 2>(p, stream);
  if (c_b < c_a) return launch_cfg<256, 256, 2, 2>(p, stream);
  return launch_cfg<256, 160, 4, 1>(p, stream);
}

}  // namespace ds
