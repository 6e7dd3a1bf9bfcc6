// Host-side launchers of the gfx950 kernels.  Every launcher checks nothing
// about pointer validity (the C ABI layer does) and enqueues on `stream`.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ds {

// Kernels that ask for more dynamic LDS than the default limit need a function attribute on every device they
// run on.  Each launcher names its (kernel, bytes) pair through KernelAttrReg, which files the pair in a
// list when the library is loaded; configure_kernels() applies the whole list to the current device.  The
// C ABI layer calls it once per device (context creation), so no launch path carries set-up state.
void register_kernel_attr(const void* fn, int lds_bytes);
hipError_t configure_kernels();
template <auto Kern, int LdsBytes>
struct KernelAttrReg {
  static inline const bool done = (register_kernel_attr(reinterpret_cast<const void*>(Kern), LdsBytes), true);
};

// y = LN(x) * gamma + beta, one workgroup per row.  h % 8 == 0, h <= 16384.
// With `row_index` (device, `rows` entries) output row r normalises input row row_index[r].
hipError_t launch_layernorm(const void* x, const void* gamma, const void* beta, void* out,
                            int rows, int h, float eps, hipStream_t stream,
                            const int32_t* row_index = nullptr);

// Epilogue of both GEMM paths: out = act(acc + bias) + residual, written as bf16.
// The N output columns may be cut into up to three segments that go to
// different buffers (Q | K | V): the first `seg_cols` wide, the other two
// `seg_cols_kv` wide (0 = as wide as the first); each buffer's row stride is
// its segment width.  Residual is only allowed with a single segment.
struct Epilogue {
  const void* bias = nullptr;      // [N] bf16 or null
  const void* residual = nullptr;  // [M, N] bf16 or null
  int relu = 0;
  void* out[3] = {nullptr, nullptr, nullptr};
  int seg_cols = 0;     // width (= row stride) of out[0]
  int seg_cols_kv = 0;  // width (= row stride) of out[1] and out[2]; 0 = seg_cols
  // Row strides other than the dense ones, in elements (multiples of 8), for the MFMA tile kernel without
  // split-K only: a row stride with many trailing zero bits (a 96 KB stride, say) lands the 128-byte pieces
  // a tile reads from consecutive rows on few memory channels, so internal buffers get 128 bytes of padding.
  int x_ld = 0;    // of X; 0 = K
  int out_ld = 0;  // of out[0], single segment only; 0 = seg_cols
};

struct SkinnyFused;

// Y[M,N] = X[M,K] W[N,K]^T (+ epilogue) on the MFMA tile kernel, any M.  Where the tiles alone
// would not fill the chip (decode-sized M, narrow N) the K axis is split over workgroups: fp32
// partials in `workspace` (gemm_workspace_bytes) and a second pass that also carries the epilogue.
// `fused` asks for extra work (see SkinnyFused); *fused_done tells whether it was carried out.
size_t gemm_workspace_bytes(int M, int N, int K);
int gemm_splits(int M, int N, int K);  // 1 = the launch will not split K
void gemm_describe(int M, int N, int K, int* tile_rows, int* tile_cols, int* splits, int* cut_cols);  // the plan launch_gemm follows
hipError_t launch_gemm(const void* X, const void* W, int M, int N, int K, const Epilogue& ep,
                       hipStream_t stream, void* workspace = nullptr, const SkinnyFused* fused = nullptr,
                       bool* fused_done = nullptr);

// Work that the decode GEMM's split-K reduction can absorb (saves a launch each):
//  kLayerNorm: after out = act(..) + residual is written, also write ln_out = LN(out) (row-wise).
//  kKvAppend : columns [0, n s) go to out[0] as usual; the next n_kv s columns and the n_kv s after
//              them are this step's K / V rows and go straight into the paged cache
//              [num_blocks, n_kv, 16, s] at position ctx_lens[row].
struct SkinnyFused {
  enum Kind { kNone = 0, kLayerNorm = 1, kKvAppend = 2 } kind = kNone;
  const void* ln_gamma = nullptr;
  const void* ln_beta = nullptr;
  float ln_eps = 0.f;
  void* ln_out = nullptr;
  const int32_t* ctx_lens = nullptr;
  const int32_t* block_tables = nullptr;
  int max_blocks = 0;
  void* k_cache = nullptr;
  void* v_cache = nullptr;
  int n_heads = 0, n_kv_heads = 0, head_dim = 0;
};

hipError_t launch_splitk_reduce(const float* partial, int splits, int M, int N, const Epilogue& ep,
                                const SkinnyFused* fused, bool* fused_done, hipStream_t stream);

// Same contraction for M <= 256 (decode): weights are streamed once from HBM.
// `*fused_done` tells whether the requested fused work was carried out (it needs the split-K
// reduction pass); if not, the caller launches the separate kernel.
size_t skinny_workspace_bytes(int M, int N, int K);
void skinny_describe(int M, int N, int K, int* tile_cols, int* splits);  // the plan launch_skinny_gemm follows
hipError_t launch_skinny_gemm(const void* X, const void* W, int M, int N, int K, const Epilogue& ep,
                              void* workspace, hipStream_t stream, const SkinnyFused* fused = nullptr,
                              bool* fused_done = nullptr);

// Greedy token choice over logits = X[M,K] W[N,K]^T (M <= 256, fp32 accumulation, never written out):
// the weight-streaming kernel keeps, per row and column block, the largest logit and its column; a
// second kernel merges the blocks (ties -> lowest column).  next_token [M] int32, best_logit [M]
// fp32 or null.  Workspace: skinny_argmax_workspace_bytes.
size_t skinny_argmax_workspace_bytes(int M, int N, int K);
hipError_t launch_skinny_argmax(const void* X, const void* W, int M, int N, int K, void* workspace,
                                int32_t* next_token, float* best_logit, hipStream_t stream);

// x[r,:] = tok_emb[clamp(token_ids[r]),:] + pos_emb[clamp(positions[r]),:] (fp32 sum, bf16 result);
// pos_emb / positions may be null (no position term).  h % 8 == 0.
hipError_t launch_embed(const int32_t* token_ids, const int32_t* positions, const void* tok_emb, int vocab,
                        const void* pos_emb, int n_pos, int rows, int h, void* x, hipStream_t stream);

// Causal attention within each packed request; q,o rows have `n_heads*head_dim` elements, k,v rows
// `n_kv_heads*head_dim` (query head j reads key/value head j / (n_heads/n_kv_heads)).
// `t` = rows in all (sum of the lengths), which only steers the choice of the workgroup order.
hipError_t launch_prefill_attention(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                                    int B, int t, int max_seqlen, int n_heads, int n_kv_heads, int head_dim, void* o,
                                    hipStream_t stream);

// contiguous [t,n,s] -> paged [num_blocks,n,16,s] for K and V in one launch
hipError_t launch_kv_migrate(const void* k_src, const void* v_src, const int32_t* cu_seqlens, int B,
                             int max_seqlen, const int32_t* block_tables, int max_blocks, void* k_cache,
                             void* v_cache, int n_heads, int head_dim, hipStream_t stream);

// new K,V rows (row stride `src_stride` elements) of B sequences -> slot ctx_lens[i] of the paged cache
hipError_t launch_kv_append(const void* k_new, const void* v_new, int src_stride, const int32_t* ctx_lens,
                            const int32_t* block_tables, int B, int max_blocks, void* k_cache, void* v_cache,
                            int n_heads, int head_dim, hipStream_t stream);

// One query per (sequence, head) over the paged cache.  kv_len_add is added to
// kv_lens[i] (1 when kv_lens holds the lengths before this step's append).
size_t decode_attention_workspace_bytes(int B, int n_heads, int n_kv_heads, int head_dim, int max_kv_len);
int decode_attention_splits(int B, int n_heads, int n_kv_heads, int head_dim, int max_kv_len);
hipError_t launch_decode_attention(const void* q, int q_stride, const int32_t* kv_lens, int kv_len_add,
                                   const int32_t* block_tables, int B, int max_blocks, int max_kv_len,
                                   const void* k_cache, const void* v_cache, int n_heads, int n_kv_heads,
                                   int head_dim, void* o, void* workspace, hipStream_t stream);

}  // namespace ds
