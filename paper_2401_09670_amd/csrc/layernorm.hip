// LayerNorm over the hidden dimension, bf16 in/out, fp32 statistics.
// One 256-thread workgroup per row; the row stays in registers between the
// mean, variance and normalise passes, so HBM sees one read and one write.
#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kLnThreads = 256;
constexpr int kLnMaxChunks = 8;  // 8 chunks x 8 elements x 256 threads = 16384 elements per row

__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// NCH = 16-byte pieces per thread (row length <= NCH * 2048 elements): the row buffer is sized to the
// row, so that short rows leave enough registers for every row of a 2048-row launch to be resident.
template <int NCH>
__global__ __launch_bounds__(kLnThreads) void layernorm_kernel(const uint16_t* __restrict__ x,
                                                               const uint16_t* __restrict__ gamma,
                                                               const uint16_t* __restrict__ beta,
                                                               uint16_t* __restrict__ out, int h, float eps,
                                                               const int32_t* __restrict__ row_index) {
  __shared__ float red[4];
  const int nchunk = h >> 3;
  const size_t row = blockIdx.x;
  // output row `row` normalises input row row_index[row] (all rows in order when there is no index)
  const uint16_t* xr = x + (row_index ? (size_t)row_index[row] : row) * (size_t)h;
  uint16_t* orow = out + row * (size_t)h;

  // Every load of the kernel is issued before anything waits: the row's pieces with their index clamped into
  // the row (a thread past the end re-reads the last piece and its values are masked out of the sums - with
  // the loads under per-thread predicates the compiler waited for each one before issuing the next, three
  // memory latencies in a row for a 5120-wide row), and the gain / shift pieces, which depend on nothing.
  u32x4 raw[NCH], g[NCH], b[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) raw[i] = ld16(xr + min((int)threadIdx.x + i * kLnThreads, nchunk - 1) * 8);
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = min((int)threadIdx.x + i * kLnThreads, nchunk - 1);
    g[i] = ld16(gamma + c * 8);
    b[i] = ld16(beta + c * 8);
  }
  float vals[NCH][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const bool live = (int)threadIdx.x + i * kLnThreads < nchunk;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      vals[i][2 * j] = bf16_lo(raw[i][j]);
      vals[i][2 * j + 1] = bf16_hi(raw[i][j]);
      sum += live ? vals[i][2 * j] + vals[i][2 * j + 1] : 0.f;
    }
  }
  const float mean = block_sum(sum, red) / (float)h;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const bool live = (int)threadIdx.x + i * kLnThreads < nchunk;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float d = vals[i][j] - mean;
      sq += live ? d * d : 0.f;
    }
  }
  const float var = block_sum(sq, red) / (float)h;
  const float rstd = rsqrtf(var + eps);
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = (int)threadIdx.x + i * kLnThreads;
    u32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float lo = (vals[i][2 * j] - mean) * rstd * bf16_lo(g[i][j]) + bf16_lo(b[i][j]);
      const float hi = (vals[i][2 * j + 1] - mean) * rstd * bf16_hi(g[i][j]) + bf16_hi(b[i][j]);
      o[j] = pack_bf16(lo, hi);
    }
    if (c < nchunk) st16(orow + c * 8, o);
  }
}

hipError_t launch_layernorm(const void* x, const void* gamma, const void* beta, void* out, int rows, int h,
                            float eps, hipStream_t stream, const int32_t* row_index) {
  if (rows <= 0) return hipSuccess;
  if (h % 8 != 0 || h > kLnThreads * 8 * kLnMaxChunks) return hipErrorInvalidValue;
  const int nch = ((h >> 3) + kLnThreads - 1) / kLnThreads;
#define DS_LN_LAUNCH(N)                                                                                   \
  hipLaunchKernelGGL(layernorm_kernel<N>, dim3(rows), dim3(kLnThreads), 0, stream, (const uint16_t*)x,   \
                     (const uint16_t*)gamma, (const uint16_t*)beta, (uint16_t*)out, h, eps, row_index)
  if (nch <= 1) DS_LN_LAUNCH(1);
  else if (nch == 2) DS_LN_LAUNCH(2);
  else if (nch == 3) DS_LN_LAUNCH(3);
  else if (nch == 4) DS_LN_LAUNCH(4);
  else if (nch <= 6) DS_LN_LAUNCH(6);
  else DS_LN_LAUNCH(8);
#undef DS_LN_LAUNCH
  return hipGetLastError();
}

}  // namespace ds
