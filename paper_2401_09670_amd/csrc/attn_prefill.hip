// Causal attention inside each packed request, flash style on the matrix cores.
//
// A workgroup (4 waves) owns 128 consecutive queries of one (request, head);
// wave w owns 32 of them.  Keys/values are visited in tiles of 64.  The score
// tile is computed transposed, S^T[key, query] = K Q^T, so that in the MFMA
// result layout every lane holds scores of ONE query (lane % 32): the running
// max / sum / rescale factors are per-lane scalars, and the probabilities are
// already in the register layout the second product O^T[d, query] = V^T P^T
// needs as its column operand - no shuffles, no LDS round trip for P.
// K is staged in LDS row-major, V transposed ([d][key]) so a lane's V^T
// fragment is two 8-byte reads.
#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kAttThreads = 256;
constexpr int kAttQ = 128;    // queries per workgroup
constexpr int kAttKV = 64;    // keys per tile
constexpr int kVtStride = kAttKV + 4;  // elements per V^T row (136 B): 8-byte reads of 16 rows hit distinct banks

template <int HD>
__global__ __launch_bounds__(kAttThreads) void prefill_attention_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_seqlens, uint16_t* __restrict__ o, int n_heads, float scale_log2e) {
  constexpr int KS = HD + 8;        // K tile row stride in elements
  constexpr int DSTEPS = HD / 16;   // MFMA k-steps over the head dimension
  constexpr int DT = HD / 32;       // 32-row tiles of O^T
  __shared__ __attribute__((aligned(16))) uint16_t ks[kAttKV * KS];
  __shared__ __attribute__((aligned(16))) uint16_t vt[HD * kVtStride];

  const int seq = blockIdx.z;
  const int head = blockIdx.y;
  const int start = cu_seqlens[seq];
  const int len = cu_seqlens[seq + 1] - start;
  // heaviest query tiles (most keys) first
  const int q0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * kAttQ;
  if (q0 >= len) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hl = lane >> 5, lq = lane & 31;
  const size_t h = (size_t)n_heads * HD;
  const uint16_t* kbase = k + (size_t)start * h + (size_t)head * HD;
  const uint16_t* vbase = v + (size_t)start * h + (size_t)head * HD;

  const int qw0 = q0 + wave * 32;  // first query of this wave
  const int my_q = qw0 + lq;
  // Q fragments (column operand of S^T = K Q^T): lane holds q[my_q][16*st + 8*hl .. +7]
  bf16x8 qf[DSTEPS];
  {
    const uint16_t* qrow = q + ((size_t)start + min(my_q, len - 1)) * h + (size_t)head * HD + hl * 8;
#pragma unroll
    for (int st = 0; st < DSTEPS; ++st) qf[st] = *reinterpret_cast<const bf16x8*>(qrow + st * 16);
  }

  floatx16 oacc[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[d][r] = 0.f;
  float m_run = -INFINITY;  // running max of raw scores for query my_q (same in lanes lq and lq+32)
  float l_run = 0.f;        // this lane's share of the running sum

  const int kv_end = min(len, q0 + kAttQ);  // keys any query of this workgroup may see
  const int n_tiles = (kv_end + kAttKV - 1) / kAttKV;

  for (int tile = 0; tile < n_tiles; ++tile) {
    const int kv0 = tile * kAttKV;
    __syncthreads();  // previous tile's LDS reads are done
    // ---- stage K tile [64][HD] row-major ----
    {
      constexpr int CPR = HD / 8;  // chunks per row
      constexpr int ITER = kAttKV * CPR / kAttThreads;
#pragma unroll
      for (int i = 0; i < ITER; ++i) {
        const int c = tid + i * kAttThreads;
        const int r = c / CPR, ch = c % CPR;
        const int key = min(kv0 + r, len - 1);
        st16(ks + r * KS + ch * 8, ld16(kbase + (size_t)key * h + ch * 8));
      }
    }
    // ---- stage V tile transposed: vt[d][key]; a thread takes two adjacent keys x 8 dims ----
    {
      constexpr int CPR = HD / 8;
      constexpr int ITEMS = (kAttKV / 2) * CPR;
      constexpr int ITER = ITEMS / kAttThreads;
#pragma unroll
      for (int i = 0; i < ITER; ++i) {
        const int c = tid + i * kAttThreads;
        const int pair = c % (kAttKV / 2), ch = c / (kAttKV / 2);
        const int key0 = min(kv0 + 2 * pair, len - 1), key1 = min(kv0 + 2 * pair + 1, len - 1);
        const u32x4 a = ld16(vbase + (size_t)key0 * h + ch * 8);
        const u32x4 b = ld16(vbase + (size_t)key1 * h + ch * 8);
        uint32_t* dst = reinterpret_cast<uint32_t*>(vt + (ch * 8) * kVtStride + 2 * pair);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          dst[(2 * j) * (kVtStride / 2)] = (a[j] & 0xffffu) | (b[j] << 16);
          dst[(2 * j + 1) * (kVtStride / 2)] = (a[j] >> 16) | (b[j] & 0xffff0000u);
        }
      }
    }
    __syncthreads();
    if (kv0 > qw0 + 31) continue;  // every key of this tile is in the future of this wave's queries

    // ---- S^T = K Q^T : two 32-key row tiles ----
    floatx16 sacc[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
      const uint16_t* kr = ks + (u * 32 + lq) * KS + hl * 8;
#pragma unroll
      for (int st = 0; st < DSTEPS; ++st) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kr + st * 16);
        sacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], sacc[u], 0, 0, 0);
      }
    }
    // ---- causal mask + running softmax; element r of tile u is key kv0 + 32u + 8(r/4) + 4hl + r%4 ----
    const bool need_mask = (kv0 + kAttKV - 1 > qw0);
    float tmax = -INFINITY;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (need_mask) {
          const int key = kv0 + u * 32 + (r >> 2) * 8 + hl * 4 + (r & 3);
          if (key > my_q) sacc[u][r] = -INFINITY;
        }
        tmax = fmaxf(tmax, sacc[u][r]);
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m_run, tmax);  // finite: key kv0=0 is visible to every query
    const float alpha = exp2f((m_run - m_new) * scale_log2e);
    const float mb = m_new * scale_log2e;
    float psum = 0.f;
    bf16x8 pf[4];  // pf[2u+v]: column operand of PV step (u,v)
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = exp2f(sacc[u][r] * scale_log2e - mb);
        psum += pv;
        pf[2 * u + (r >> 3)][r & 7] = (__bf16)pv;
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[d][r] *= alpha;

    // ---- O^T += V^T P^T.  PV step (u,v) contracts keys 32u+16v + {0..3, 8..11} + 4hl ----
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int vv = 0; vv < 2; ++vv) {
        const int kb = u * 32 + vv * 16 + hl * 4;
#pragma unroll
        for (int d = 0; d < DT; ++d) {
          const uint16_t* vr = vt + (d * 32 + lq) * kVtStride + kb;
          const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vr);
          const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vr + 8);
          bf16x8 vf;
          vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
          vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
          oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[2 * u + vv], oacc[d], 0, 0, 0);
        }
      }
  }

  // ---- normalise and store: lane holds O[my_q][32d + 8g + 4hl + i] ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (my_q < len) {
    const float inv = 1.f / l_tot;
    uint16_t* orow = o + ((size_t)start + my_q) * h + (size_t)head * HD + hl * 4;
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16(oacc[d][4 * g] * inv, oacc[d][4 * g + 1] * inv);
        w[1] = pack_bf16(oacc[d][4 * g + 2] * inv, oacc[d][4 * g + 3] * inv);
        *reinterpret_cast<u32x2*>(orow + d * 32 + g * 8) = w;
      }
  }
}

hipError_t launch_prefill_attention(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                                    int B, int max_seqlen, int n_heads, int head_dim, void* o,
                                    hipStream_t stream) {
  if (B <= 0 || max_seqlen <= 0) return hipSuccess;
  if (B > 65535 || n_heads > 65535) return hipErrorInvalidValue;
  const dim3 grid((max_seqlen + kAttQ - 1) / kAttQ, n_heads, B);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
  if (head_dim == 128) {
    hipLaunchKernelGGL(prefill_attention_kernel<128>, grid, dim3(kAttThreads), 0, stream, (const uint16_t*)q,
                       (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, (uint16_t*)o, n_heads, scale_log2e);
  } else if (head_dim == 64) {
    hipLaunchKernelGGL(prefill_attention_kernel<64>, grid, dim3(kAttThreads), 0, stream, (const uint16_t*)q,
                       (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, (uint16_t*)o, n_heads, scale_log2e);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ds
