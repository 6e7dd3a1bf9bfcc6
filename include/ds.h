/*
 * ds.h — C ABI of the MI355X (gfx950) prefill / KV-migrate / decode library.
 *
 * The library computes, for ONE transformer layer of an OPT-style decoder
 * (pre-LayerNorm, ReLU FFN, multi-head attention; paper Sec. 6.1 / App. A):
 *   - the prefill pass over packed prompts      (App. A.2: QKV, Attn-Output,
 *     FFN-Input, FFN-Output GEMMs + per-request causal attention),
 *   - the decode step over a paged KV cache     (App. A.3: the same four GEMMs
 *     at B rows + one-query attention over the cached tokens),
 *   - the KV hand-off from the prefill side's contiguous K/V to the decode
 *     side's paged block layout                 (Sec. 3.3, Sec. 4.3 "pull").
 * The caller loops over layers.  Symbols follow App. A.1: h hidden size,
 * n heads, s head size (h = n*s), m FFN size, B batch, l_i lengths, t = sum l_i.
 *
 * Conventions that hold for every call:
 *   - "device" pointers are HIP device memory, 16-byte aligned, caller-owned;
 *     the library never allocates, frees or keeps them past the call.
 *   - bf16 tensors are row-major; accumulation is fp32.
 *   - Matrices are [out_features, in_features] (reduction dim contiguous).
 *     w_qkv rows are [Q | K | V]; inside each third row = head*s + d.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream); no call synchronises; outputs are valid once the
 *     caller has synchronised the stream.
 *   - Calls record kernel launches only (no allocation, host copy or memset), so a
 *     sequence of calls can be captured into a HIP graph.  Kernel attributes are
 *     set once per device by ds_create (or by the first call on a device the
 *     context was not created on), never on a launch path.  A context is not
 *     thread-safe: one thread at a time per ds_ctx.
 *   - Errors are returned as ds_status; arguments are checked on the host
 *     before anything is launched.  Contents of device index arrays
 *     (cu_seqlens, block_tables, ctx_lens / kv_lens) are NOT validated by default
 *     (that needs a copy to the host and a stream synchronisation): out-of-range
 *     entries are the caller's responsibility, and a max_ctx / max_seqlen bound
 *     smaller than a real length silently drops the excess tokens.  The debug
 *     path - DS_DEBUG_VALIDATE=1 in the environment when the context is created,
 *     or ds_set_validate(ctx, 1) - copies these arrays back before launching and
 *     returns DS_ERR_BOUNDS naming the first offending entry; it synchronises the
 *     stream, so it must not be used under graph capture.  ds_last_error() gives
 *     text.
 *   - Paged cache layout: k_cache, v_cache [num_blocks, n, block_size, s] bf16.
 *     Token j of sequence i lives in block block_tables[i*max_blocks + j/bs],
 *     slot j % bs.  Unused table entries are -1 and never dereferenced.
 */
#ifndef DS_H_
#define DS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DS_OK = 0,
  DS_ERR_INVALID_ARG = 1, /* NULL / non-positive size / misaligned pointer / inconsistent sizes */
  DS_ERR_UNSUPPORTED = 2, /* a shape this build has no kernel for */
  DS_ERR_WORKSPACE = 3,   /* workspace smaller than ds_*_workspace_bytes() */
  DS_ERR_HIP = 4,         /* a HIP runtime call or launch failed */
  DS_ERR_BOUNDS = 5       /* debug validation: an entry of a device index array is out of range */
} ds_status;

/* Layer dimensions.  Supported: head_dim in {64,128}; hidden = n_heads*head_dim;
 * hidden and ffn multiples of 64; block_size = 16.  n_kv_heads (0 = n_heads) is the
 * number of key/value heads n_kv; with n_kv < n (n % n_kv == 0: grouped-query
 * attention, which Sec. 3.2 names as a way to shrink the KV cache) query head j
 * uses key/value head j / (n/n_kv), and wherever this header writes "n" for a K or
 * V tensor (k_out, v_out, the paged caches) n_kv is meant; w_qkv is
 * [(n + 2 n_kv) s, h] with rows [Q | K | V]. */
typedef struct {
  int32_t hidden;     /* h */
  int32_t n_heads;    /* n */
  int32_t head_dim;   /* s */
  int32_t ffn;        /* m */
  int32_t block_size; /* tokens per KV page */
  float ln_eps;       /* LayerNorm epsilon (biased variance, fp32 statistics) */
  int32_t n_kv_heads; /* n_kv; 0 means n_heads */
} ds_model_cfg;

/* One layer's parameters: device pointers to bf16.  Bias pointers may be NULL
 * (= no bias).  LayerNorm gain/shift must be present. */
typedef struct {
  const void *ln1_g, *ln1_b;   /* [h] */
  const void *w_qkv, *b_qkv;   /* [3h,h], [3h] */
  const void *w_o, *b_o;       /* [h,h],  [h]  */
  const void *ln2_g, *ln2_b;   /* [h] */
  const void *w_fc1, *b_fc1;   /* [m,h],  [m]  */
  const void *w_fc2, *b_fc2;   /* [h,m],  [h]  */
} ds_layer_weights;

typedef struct ds_ctx ds_ctx; /* opaque; owns no device memory */

/* Create / destroy a context for one layer shape on the current HIP device. */
ds_status ds_create(const ds_model_cfg *cfg, ds_ctx **out);
void ds_destroy(ds_ctx *ctx);
/* Text of the last error recorded on ctx (never NULL). */
const char *ds_last_error(const ds_ctx *ctx);
/* Turn the debug validation of device index arrays on / off (see the conventions above).  When on,
 * ds_prefill, ds_prefill_attention and ds_kv_migrate check cu_seqlens (starts at 0, ends at t, every
 * length in [1, max_seqlen]); ds_kv_migrate, ds_decode_step and ds_decode_attention check that every
 * page a sequence's tokens need is named in block_tables with an id in [0, num_blocks), and that
 * ctx_lens[i] + 1 lies in [1, max_ctx] (kv_lens[i] in [0, max_kv_len]). */
ds_status ds_set_validate(ds_ctx *ctx, int32_t on);

/* Workspace (device bytes) ds_prefill needs for up to max_tokens packed tokens.
 * Both sizes are upper bounds over all smaller calls: a workspace sized for the
 * largest batch serves every call with fewer tokens / sequences / cached tokens. */
size_t ds_prefill_workspace_bytes(const ds_ctx *ctx, int32_t max_tokens);
/* Workspace ds_decode_step needs for up to max_batch sequences of up to max_ctx cached tokens. */
size_t ds_decode_workspace_bytes(const ds_ctx *ctx, int32_t max_batch, int32_t max_ctx);

/*
 * Prefill (App. A.2): one layer over B packed prompts.
 *   x          device [t,h] bf16, row r = token r of the packed batch
 *   cu_seqlens device [B+1] int32, cu[0]=0, cu[B]=t (prompt i = rows cu[i]..cu[i+1]-1)
 *   max_seqlen host upper bound of the prompt lengths (sizes the attention grid)
 *   y          device [t,h] bf16 layer output; must not alias x
 *   k_out,v_out device [t,n,s] bf16: this layer's K,V rows, contiguous per token
 *              (what the prefill instance keeps until the decode side pulls it)
 */
ds_status ds_prefill(ds_ctx *ctx, const ds_layer_weights *w, const void *x,
                     const int32_t *cu_seqlens, int32_t B, int32_t t, int32_t max_seqlen,
                     void *y, void *k_out, void *v_out,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * KV hand-off (Sec. 3.3 / 4.3): scatter contiguous K,V rows of B prompts into
 * the paged cache.  Pure byte copy (bit-exact).  Slots no token maps to, and
 * blocks not named in block_tables, are left untouched.
 *   k_src,v_src  device [t,n,s] bf16 (ds_prefill's k_out, v_out)
 *   block_tables device [B,max_blocks_per_seq] int32
 *   max_seqlen   host upper bound of the prompt lengths
 */
ds_status ds_kv_migrate(ds_ctx *ctx, const void *k_src, const void *v_src,
                        const int32_t *cu_seqlens, int32_t B, int32_t t, int32_t max_seqlen,
                        const int32_t *block_tables, int32_t max_blocks_per_seq,
                        void *k_cache, void *v_cache, int32_t num_blocks, void *stream);

/*
 * Decode step (App. A.3): one new token for each of B sequences.
 *   x        device [B,h] bf16 new-token activations
 *   ctx_lens device [B] int32: tokens already cached BEFORE this step.  The new
 *            token's K,V are appended at position ctx_lens[i] (its page must
 *            already be present in block_tables) and the query attends over
 *            ctx_lens[i]+1 keys.  The caller increments ctx_lens between steps.
 *   max_ctx  host upper bound of ctx_lens[i]+1 (sizes the split of the KV axis)
 *   y        device [B,h] bf16; must not alias x
 * Cache slots past a sequence's last token (the rest of its last page) may hold
 * any bit pattern, NaN included: they never reach a result.
 */
ds_status ds_decode_step(ds_ctx *ctx, const ds_layer_weights *w, const void *x,
                         const int32_t *ctx_lens, const int32_t *block_tables,
                         int32_t B, int32_t max_blocks_per_seq, int32_t max_ctx,
                         void *k_cache, void *v_cache, int32_t num_blocks,
                         void *y, void *workspace, size_t workspace_bytes, void *stream);

/*
 * ds_decode_step for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * same results as ds_decode_step, minus the workspace: the step's scratch (activations between its
 * kernels, split-K and attention partial sums) lives in a static device array of DS_STATIC_SCRATCH_BYTES
 * that every GPU the library runs on holds until the process ends.  The call allocates and frees nothing.
 * A step that needs more (ds_decode_workspace_bytes(ctx, B, max_ctx) > DS_STATIC_SCRATCH_BYTES, e.g.
 * batches beyond ~128 sequences of an OPT-13B layer) is rejected with DS_ERR_WORKSPACE before anything is
 * launched.  All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different
 * streams, different threads or contexts) race on it and must be serialised by the caller; nothing in the
 * array has to survive from one call to the next, and nothing in it has to start out as zero.
 */
#define DS_STATIC_SCRATCH_BYTES (32u << 20)
ds_status ds_decode_step_static(ds_ctx *ctx, const ds_layer_weights *w, const void *x,
                                const int32_t *ctx_lens, const int32_t *block_tables,
                                int32_t B, int32_t max_blocks_per_seq, int32_t max_ctx,
                                void *k_cache, void *v_cache, int32_t num_blocks,
                                void *y, void *stream);

/* ---- the individual steps, exported for per-kernel parity tests and timing ---- */

/* out[r,:] = LN(x[r,:]) * gamma + beta, rows x h bf16 (App. A: LayerNorm is a
 * memory-bound op beside the GEMMs). */
ds_status ds_layernorm(ds_ctx *ctx, const void *x, const void *gamma, const void *beta,
                       int32_t rows, void *out, void *stream);

/* y[rows,out_f] = act(x[rows,in_f] w[out_f,in_f]^T + bias) + residual   (GEMM tables
 * of App. A.2 / A.3).  bias, residual may be NULL; relu != 0 applies max(0,.)
 * before the residual.  in_f % 64 == 0, out_f % 8 == 0.  Few rows take the
 * weight-streaming kernels of the decode phase, many the MFMA tile kernel; either
 * may split the reduction over workgroups and then needs `workspace` of
 * ds_linear_workspace_bytes(rows, ...) bytes for fp32 partial sums (0 = none
 * needed for this shape). */
size_t ds_linear_workspace_bytes(const ds_ctx *ctx, int32_t rows, int32_t in_f, int32_t out_f);
/* Which kernel a ds_linear call of this shape takes (host-side planning only, nothing is launched):
 * *streaming = 1 for the weight-streaming kernels of the decode phase (then tile_rows = 0 and tile_cols =
 * output columns per workgroup), 0 for the MFMA tile kernel with tiles of tile_rows x tile_cols outputs;
 * *splits = workgroups the
 * reduction dimension is split over (1 = not split; a split launch is followed by a reduce pass);
 * *cut_cols > 0 = the output columns from there on run as a second launch on a smaller tile.
 * App. A.2 / A.3 give the product shapes; the plan is this library's answer to how many tokens it takes
 * to fill the chip (Sec. 3.1). */
ds_status ds_linear_plan(const ds_ctx *ctx, int32_t rows, int32_t in_f, int32_t out_f, int32_t *streaming,
                         int32_t *tile_rows, int32_t *tile_cols, int32_t *splits, int32_t *cut_cols);
ds_status ds_linear(ds_ctx *ctx, const void *x, const void *w, const void *bias,
                    const void *residual, int32_t relu, int32_t rows, int32_t in_f, int32_t out_f,
                    void *y, void *workspace, size_t workspace_bytes, void *stream);

/* ---- the two ends of the token loop around the layer stack ----
 * Sec. 2.1 describes the loop these close: the prompt's tokens enter the layer
 * stack, the prefill pass yields the first new token, each decoding step one
 * more.  Neither call belongs to a layer; the caller runs ds_embed before the
 * first layer and ds_next_token after the last. */

/* x[r,:] = tok_emb[token_ids[r],:] + pos_emb[positions[r],:]   (fp32 sum, bf16
 * result; OPT, the model family of Sec. 6.1, uses a learned position table).
 * token_ids, positions: device int32 [rows]; tok_emb device bf16 [vocab,h];
 * pos_emb device bf16 [n_pos,h] or NULL (then positions may be NULL and no
 * position row is added); x device bf16 [rows,h].  Ids outside the tables are
 * clamped into them (never a wild read). */
ds_status ds_embed(ds_ctx *ctx, const int32_t *token_ids, const int32_t *positions,
                   const void *tok_emb, int32_t vocab, const void *pos_emb, int32_t n_pos,
                   int32_t rows, void *x, void *stream);

/* Greedy choice of the next token for `rows` (<= 256) hidden rows:
 *   a = LN(x[row_index[r],:]; ln_g, ln_b)  (bf16, as inside a layer),
 *   logits[r,:] = a w_vocab^T              (fp32 accumulation, never stored),
 *   next_token[r] = argmax over the vocab, ties -> lowest id.
 * x device bf16 [x_rows,h]; row_index device int32 [rows] or NULL (rows 0..rows-1):
 * after a packed prefill the last position of each prompt, cu_seqlens[i+1]-1;
 * w_vocab device bf16 [vocab,h] (OPT ties it to tok_emb); vocab % 8 == 0;
 * next_token device int32 [rows]; best_logit device fp32 [rows] or NULL.
 * Entries of row_index are not validated. */
size_t ds_next_token_workspace_bytes(const ds_ctx *ctx, int32_t rows, int32_t vocab);
ds_status ds_next_token(ds_ctx *ctx, const void *x, const int32_t *row_index, int32_t rows,
                        const void *ln_g, const void *ln_b, const void *w_vocab, int32_t vocab,
                        int32_t *next_token, float *best_logit, void *workspace,
                        size_t workspace_bytes, void *stream);

/* Per-request causal attention over packed q,k,v [t,n,s] -> o [t,n,s] (App. A.2). */
ds_status ds_prefill_attention(ds_ctx *ctx, const void *q, const void *k, const void *v,
                               const int32_t *cu_seqlens, int32_t B, int32_t t, int32_t max_seqlen,
                               void *o, void *stream);

/* One-query attention over the paged cache: sequence i attends over its first
 * kv_lens[i] cached tokens (App. A.3).  q,o device [B,n,s]; max_kv_len is a host
 * bound of kv_lens; workspace of ds_decode_workspace_bytes(B, max_kv_len).  A sequence
 * with kv_lens[i] = 0 has nothing to attend over: its output rows are 0. */
ds_status ds_decode_attention(ds_ctx *ctx, const void *q, const int32_t *kv_lens,
                              const int32_t *block_tables, int32_t B, int32_t max_blocks_per_seq,
                              int32_t max_kv_len, const void *k_cache, const void *v_cache,
                              int32_t num_blocks, void *o,
                              void *workspace, size_t workspace_bytes, void *stream);

/* ---- per-kernel timing (HIP events around every launch; off by default) ---- */
enum {
  DS_K_LAYERNORM = 0, DS_K_GEMM = 1, DS_K_PREFILL_ATTN = 2, DS_K_KV_MIGRATE = 3,
  DS_K_SKINNY_GEMM = 4 /* incl. its split-K reduce */, DS_K_DECODE_ATTN = 5 /* incl. split merge */,
  DS_K_KV_APPEND = 6, DS_K_TOKEN_IO = 7 /* embedding gather; the logits GEMM + greedy-choice merge */,
  DS_K_COUNT = 8
};
/* Turn timing on/off.  When on, every launch is bracketed by events on the
 * caller's stream (this serialises nothing, but adds event overhead). */
ds_status ds_profile_enable(ds_ctx *ctx, int32_t on);
/* Synchronise the recorded events, add their durations per kernel class into
 * ms[DS_K_COUNT] / launches[DS_K_COUNT], and clear the record. */
ds_status ds_profile_collect(ds_ctx *ctx, double *ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* DS_H_ */
