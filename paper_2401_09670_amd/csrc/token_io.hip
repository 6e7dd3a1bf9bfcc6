// The two ends of the token loop around the layer stack (Sec. 2.1: a prompt's tokens go in, the
// prefill pass produces the first new token, every decoding step one more): the embedding gather on
// the way in; on the way out the merge of the per-column-block maxima that the logits GEMM leaves.
#include <limits.h>

#include "common.h"
#include "kernels.h"

namespace ds {

// One workgroup per output row, 16-byte pieces.  Ids outside the tables are clamped into them (a
// wrong id must not become a wild read).
__global__ __launch_bounds__(256) void embed_kernel(const int32_t* __restrict__ token_ids,
                                                    const int32_t* __restrict__ positions,
                                                    const uint16_t* __restrict__ tok_emb, int vocab,
                                                    const uint16_t* __restrict__ pos_emb, int n_pos, int h,
                                                    uint16_t* __restrict__ x) {
  const size_t row = blockIdx.x;
  const int id = min(max(token_ids[row], 0), vocab - 1);
  const uint16_t* te = tok_emb + (size_t)id * h;
  const uint16_t* pe = nullptr;
  if (pos_emb) pe = pos_emb + (size_t)min(max(positions[row], 0), n_pos - 1) * h;
  uint16_t* xr = x + row * (size_t)h;
  for (int c = threadIdx.x; c < (h >> 3); c += 256) {
    u32x4 a = ld16(te + c * 8);
    if (pe) {
      const u32x4 b = ld16(pe + c * 8);
#pragma unroll
      for (int j = 0; j < 4; ++j) a[j] = pack_bf16(bf16_lo(a[j]) + bf16_lo(b[j]), bf16_hi(a[j]) + bf16_hi(b[j]));
    }
    st16(xr + c * 8, a);
  }
}

hipError_t launch_embed(const int32_t* token_ids, const int32_t* positions, const void* tok_emb, int vocab,
                        const void* pos_emb, int n_pos, int rows, int h, void* x, hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  if (h % 8 != 0 || vocab <= 0 || (pos_emb && (n_pos <= 0 || !positions))) return hipErrorInvalidValue;
  hipLaunchKernelGGL(embed_kernel, dim3(rows), dim3(256), 0, stream, token_ids, positions,
                     (const uint16_t*)tok_emb, vocab, (const uint16_t*)pos_emb, n_pos, h, (uint16_t*)x);
  return hipGetLastError();
}

// Merge the column blocks' candidates of one row: largest value, lowest column among equals.
// part_val / part_idx are [n_blocks][M].
__global__ __launch_bounds__(64) void argmax_merge_kernel(const float* __restrict__ part_val,
                                                          const int32_t* __restrict__ part_idx, int n_blocks,
                                                          int M, int32_t* __restrict__ next_token,
                                                          float* __restrict__ best_logit) {
  const int m = blockIdx.x;
  float bv = -INFINITY;
  int bi = INT_MAX;
  for (int b = threadIdx.x; b < n_blocks; b += 64) {
    const float v = part_val[(size_t)b * M + m];
    const int i = part_idx[(size_t)b * M + m];
    if (v > bv || (v == bv && i < bi)) {
      bv = v;
      bi = i;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    if (ov > bv || (ov == bv && oi < bi)) {
      bv = ov;
      bi = oi;
    }
  }
  if (threadIdx.x == 0) {
    next_token[m] = bi;
    if (best_logit) best_logit[m] = bv;
  }
}

hipError_t launch_argmax_merge(const float* part_val, const int32_t* part_idx, int n_blocks, int M,
                               int32_t* next_token, float* best_logit, hipStream_t stream) {
  hipLaunchKernelGGL(argmax_merge_kernel, dim3(M), dim3(64), 0, stream, part_val, part_idx, n_blocks, M,
                     next_token, best_logit);
  return hipGetLastError();
}

}  // namespace ds
