// Decode-phase GEMM: Y[M,N] = act(X[M,K] W[N,K]^T + bias) + residual, M <= 256.
// The weights (N*K*2 bytes) are read once from HBM and dominate the traffic
// (App. A.3: 4h^2 + 2hm elements per layer), so the kernel is organised
// around streaming W: every wave pulls its own 16 weight rows straight from
// global memory into MFMA fragments (no LDS hop for the big operand), while
// the small activation slab X[:, k..k+128) is staged once per workgroup in LDS
// and shared by the four waves.
//
// grid = (N/64, KSPLIT).  Workgroup = 4 waves; wave w owns weight rows
// n0+16w .. n0+16w+15 and all M activation rows (M/16 MFMA 16x16x32 tiles).
// The tile is computed transposed (weights as MFMA row operand), so a lane
// ends up with 4 consecutive output columns of one row.  With KSPLIT > 1 each
// split writes fp32 partial sums and a second kernel reduces them in a fixed
// order and applies the epilogue.
#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kSkThreads = 256;
constexpr int kSkBN = 64;                 // weight rows per workgroup
constexpr int kSkKS = 128;                // k elements per slab
constexpr int kSkXStride = kSkKS + 8;     // LDS row stride (272 B) for conflict-free 16-byte reads
constexpr int kSkSteps = kSkKS / 32;      // MFMA k-steps per slab

struct SkinnyParams {
  const uint16_t* X;
  const uint16_t* W;
  const uint16_t* bias;
  const uint16_t* residual;
  uint16_t* out[3];
  int seg_cols;
  int M, N, K;
  int relu;
  int slabs_per_split;
  float* partial;  // [KSPLIT][M][N] fp32 when gridDim.y > 1
};

template <int MT>  // activation row tiles of 16
__global__ __launch_bounds__(kSkThreads) void skinny_gemm_kernel(const SkinnyParams p) {
  constexpr int MP = MT * 16;                       // padded rows held in LDS
  constexpr int XCH = MP * (kSkKS / 8) / kSkThreads;  // 16-byte chunks per thread per slab (= MT)
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];  // [2][MP][kSkXStride]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * kSkBN;
  const int split = blockIdx.y;
  const int slabs_total = p.K / kSkKS;
  const int slab_lo = split * p.slabs_per_split;
  const int slab_hi = min(slabs_total, slab_lo + p.slabs_per_split);
  const int ns = slab_hi - slab_lo;
  const int K = p.K;

  uint32_t xoff[XCH], xlds[XCH];
#pragma unroll
  for (int i = 0; i < XCH; ++i) {
    const int c = tid + i * kSkThreads;
    const int r = c >> 4, kc = c & 15;
    xoff[i] = (uint32_t)min(r, p.M - 1) * (uint32_t)K + kc * 8;
    xlds[i] = r * kSkXStride + kc * 8;
  }
  const int wrow = min(n0 + wave * 16 + (lane & 15), p.N - 1);
  const uint16_t* Wp = p.W + (size_t)wrow * K + (size_t)slab_lo * kSkKS + (lane >> 4) * 8;
  const uint16_t* Xp = p.X + (size_t)slab_lo * kSkKS;

  floatx4 acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};

  u32x4 xr[XCH];
  bf16x8 wcur[kSkSteps], wnext[kSkSteps];
  auto gload_x = [&]() {
#pragma unroll
    for (int i = 0; i < XCH; ++i) xr[i] = ld16(Xp + xoff[i]);
    Xp += kSkKS;
  };
  auto gload_w = [&](bf16x8* dst) {
#pragma unroll
    for (int s = 0; s < kSkSteps; ++s) dst[s] = *reinterpret_cast<const bf16x8*>(Wp + s * 32);
    Wp += kSkKS;
  };
  auto sstore = [&](int buf) {
    uint16_t* xb = lds + buf * MP * kSkXStride;
#pragma unroll
    for (int i = 0; i < XCH; ++i) st16(xb + xlds[i], xr[i]);
  };

  if (ns > 0) {
    gload_x();
    gload_w(wcur);
    sstore(0);
  }
  __syncthreads();
  for (int i = 0; i < ns; ++i) {
    const int buf = i & 1;
    if (i + 1 < ns) {
      gload_x();
      gload_w(wnext);
    }
    const uint16_t* xb = lds + buf * MP * kSkXStride + (lane & 15) * kSkXStride + (lane >> 4) * 8;
#pragma unroll
    for (int s = 0; s < kSkSteps; ++s) {
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const bf16x8 xf = *reinterpret_cast<const bf16x8*>(xb + t * 16 * kSkXStride + s * 32);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wcur[s], xf, acc[t], 0, 0, 0);
      }
    }
    if (i + 1 < ns) {
      sstore(buf ^ 1);
#pragma unroll
      for (int s = 0; s < kSkSteps; ++s) wcur[s] = wnext[s];
    }
    __syncthreads();
  }

  // acc[t][r]: row m = 16t + lane%16, column n = n0 + 16*wave + 4*(lane/16) + r
  const int n = n0 + wave * 16 + (lane >> 4) * 4;
  if (n >= p.N) return;
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int m = t * 16 + (lane & 15);
    if (m >= p.M) continue;
    if (gridDim.y > 1) {
      *reinterpret_cast<floatx4*>(p.partial + ((size_t)split * p.M + m) * p.N + n) = acc[t];
      continue;
    }
    float v0 = acc[t][0], v1 = acc[t][1], v2 = acc[t][2], v3 = acc[t][3];
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
    const int seg = n / p.seg_cols;
    const int col = n - seg * p.seg_cols;
    u32x2 ov;
    ov[0] = pack_bf16(v0, v1);
    ov[1] = pack_bf16(v2, v3);
    *reinterpret_cast<u32x2*>(p.out[seg] + (size_t)m * p.seg_cols + col) = ov;
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
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float* src = p.partial + ((size_t)s * p.M + m) * p.N + n;
    const floatx4 a = *reinterpret_cast<const floatx4*>(src);
    const floatx4 b = *reinterpret_cast<const floatx4*>(src + 4);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[j] += a[j];
      v[4 + j] += b[j];
    }
  }
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
  const int seg = n / p.seg_cols;
  const int col = n - seg * p.seg_cols;
  u32x4 ov;
#pragma unroll
  for (int j = 0; j < 4; ++j) ov[j] = pack_bf16(v[2 * j], v[2 * j + 1]);
  st16(p.out[seg] + (size_t)m * p.seg_cols + col, ov);
}

// Split the K axis until about two workgroups per CU exist, keeping >= 4 slabs per split.
static int skinny_splits(int N, int K) {
  const int wgs = (N + kSkBN - 1) / kSkBN;
  const int slabs = K / kSkKS;
  int splits = (2 * 256 + wgs - 1) / wgs;
  const int max_splits = slabs / 4 > 0 ? slabs / 4 : 1;
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  const int per = (slabs + splits - 1) / splits;
  return (slabs + per - 1) / per;  // drop empty splits
}

size_t skinny_workspace_bytes(int M, int N, int K) {
  if (K % kSkKS != 0) return 0;
  const int splits = skinny_splits(N, K);
  return splits > 1 ? (size_t)splits * M * N * sizeof(float) : 0;
}

template <int MT>
static hipError_t launch_skinny_mt(const SkinnyParams& p, int splits, hipStream_t stream) {
  constexpr size_t lds_bytes = 2ull * MT * 16 * kSkXStride * sizeof(uint16_t);
  auto kern = skinny_gemm_kernel<MT>;
  static bool attr_set = false;
  if (!attr_set && lds_bytes > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((p.N + kSkBN - 1) / kSkBN, splits), dim3(kSkThreads), lds_bytes, stream, p);
  return hipGetLastError();
}

hipError_t launch_skinny_gemm(const void* X, const void* W, int M, int N, int K, const Epilogue& ep,
                              void* workspace, hipStream_t stream) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (M > 256 || K % kSkKS != 0 || N % 8 != 0 || ep.seg_cols <= 0 || ep.seg_cols % 8 != 0)
    return hipErrorInvalidValue;
  SkinnyParams p;
  p.X = (const uint16_t*)X;
  p.W = (const uint16_t*)W;
  p.bias = (const uint16_t*)ep.bias;
  p.residual = (const uint16_t*)ep.residual;
  for (int i = 0; i < 3; ++i) p.out[i] = (uint16_t*)ep.out[i];
  p.seg_cols = ep.seg_cols;
  p.M = M; p.N = N; p.K = K;
  p.relu = ep.relu;
  const int splits = skinny_splits(N, K);
  const int slabs = K / kSkKS;
  p.slabs_per_split = (slabs + splits - 1) / splits;
  p.partial = (float*)workspace;
  if (splits > 1 && workspace == nullptr) return hipErrorInvalidValue;
  hipError_t e;
  const int mt = (M + 15) / 16;
  if (mt <= 1) e = launch_skinny_mt<1>(p, splits, stream);
  else if (mt <= 2) e = launch_skinny_mt<2>(p, splits, stream);
  else if (mt <= 4) e = launch_skinny_mt<4>(p, splits, stream);
  else if (mt <= 8) e = launch_skinny_mt<8>(p, splits, stream);
  else e = launch_skinny_mt<16>(p, splits, stream);
  if (e != hipSuccess) return e;
  if (splits > 1) {
    const long items = (long)M * (N / 8);
    hipLaunchKernelGGL(skinny_reduce_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, stream, p,
                       splits);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace ds
