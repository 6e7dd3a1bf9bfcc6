// C ABI of the library (declared in include/ds.h): argument checks on the
// host, workspace carving, and the order in which the kernels of one layer
// are enqueued.  No device memory is allocated here.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "../../include/ds.h"
#include "kernels.h"

struct ds_ctx {
  ds_model_cfg cfg;  // n_kv_heads is normalised at creation: always the actual count, never 0
  char err[512];
  bool profile;
  bool validate;  // copy the index arrays back and check them before launching (debug path)
  struct Rec {
    int kind;
    hipEvent_t a, b;
  };
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  // Workspace sizes already worked out (they walk every smaller row count through the GEMM planners, tens of
  // microseconds; every ds_prefill / ds_decode_step call checks its workspace against them).
  mutable std::map<int, size_t> prefill_ws;
  mutable std::map<std::pair<int, int>, size_t> decode_ws;
};

// ---- per-device set-up: kernel attributes, address of the static scratch array ----
namespace ds {
namespace {
std::vector<std::pair<const void*, int>>& attr_list() {
  static std::vector<std::pair<const void*, int>> list;
  return list;
}
}  // namespace
void register_kernel_attr(const void* fn, int lds_bytes) { attr_list().emplace_back(fn, lds_bytes); }
hipError_t configure_kernels() {
  for (const auto& a : attr_list()) {
    const hipError_t e = hipFuncSetAttribute(a.first, hipFuncAttributeMaxDynamicSharedMemorySize, a.second);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
}  // namespace ds

// Scratch of ds_decode_step_static: the decode step's workspace (activations between its kernels, split-K
// and attention partials) for callers that cannot bring one.  One copy per GPU the library runs on, held
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress: kernels and
// copies are given the per-device address kept in DeviceState::scratch, never the name.
static __device__ __align__(256) unsigned char scratch[DS_STATIC_SCRATCH_BYTES];

#ifdef DS_DEV_SWITCHES
#include "common.h"
// Development builds: the planning switches by name (the sweep harness sets them through ds_dev_switch).
namespace ds {
namespace {
struct SwitchEntry {
  const char* name;
  int* value;
};
std::vector<SwitchEntry>& switch_table() {
  static std::vector<SwitchEntry> t;
  return t;
}
}  // namespace
SwitchReg::SwitchReg(const char* name, int* value) { switch_table().push_back({name, value}); }
}  // namespace ds

// Sets switch `name` to `value`; returns its previous value, or INT32_MIN if there is no such switch.
extern "C" int32_t ds_dev_switch(const char* name, int32_t value) {
  for (auto& e : ds::switch_table())
    if (strcmp(e.name, name) == 0) {
      const int32_t old = *e.value;
      *e.value = value;
      return old;
    }
  return INT32_MIN;
}
#endif

namespace {

constexpr int kMaxDevices = 64;
struct DeviceState {
  bool ready = false;
  void* scratch = nullptr;  // this device's address of `scratch`
};
std::mutex g_dev_mu;
DeviceState g_dev[kMaxDevices];

// Once per device, with that device current: function attributes of every kernel, and the device address
// of `scratch` (each GPU holds its own copy of the array at its own address).  Returns the device's state,
// or null with *err set.
const DeviceState* device_state(hipError_t* err) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
  if (e != hipSuccess) {
    *err = e;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_dev_mu);
  DeviceState& st = g_dev[dev];
  if (!st.ready) {
    e = ds::configure_kernels();
    void* ptr = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      *err = e != hipSuccess ? e : hipErrorInvalidSymbol;
      return nullptr;
    }
    st.scratch = ptr;
    st.ready = true;
  }
  *err = hipSuccess;
  return &st;
}

constexpr int kSkinnyMaxRows = 256;

// widths of the K/V rows and of the QKV projection output: n_kv s and (n + 2 n_kv) s
int kv_width(const ds_model_cfg& c) { return c.n_kv_heads * c.head_dim; }
int qkv_width(const ds_model_cfg& c) { return c.hidden + 2 * kv_width(c); }

ds_status fail(ds_ctx* ctx, ds_status st, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Brackets one launcher call with events when profiling is on.
struct Timed {
  ds_ctx* ctx;
  hipStream_t stream;
  int kind;
  hipEvent_t a = nullptr, b = nullptr;
  Timed(ds_ctx* c, hipStream_t s, int k) : ctx(c), stream(s), kind(k) {
    if (!ctx->profile) return;
    a = take();
    b = take();
    if (a && b) {
      (void)hipEventRecord(a, stream);
    } else {  // no timing for this launch; an event that was obtained goes back to the pool
      if (a) ctx->pool.push_back(a);
      if (b) ctx->pool.push_back(b);
      a = b = nullptr;
    }
  }
  ~Timed() {
    if (!ctx->profile || !a || !b) return;
    (void)hipEventRecord(b, stream);
    ctx->recs.push_back({kind, a, b});
  }
  hipEvent_t take() {
    if (!ctx->pool.empty()) {
      hipEvent_t e = ctx->pool.back();
      ctx->pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};

#define DS_LAUNCH(ctx, stream, kind, call)                                              \
  do {                                                                                  \
    hipError_t e_;                                                                      \
    {                                                                                   \
      Timed t_(ctx, stream, kind);                                                      \
      e_ = (call);                                                                      \
    }                                                                                   \
    if (e_ != hipSuccess)                                                               \
      return fail(ctx, DS_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));      \
  } while (0)

struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* p) : base(static_cast<char*>(p)) {}
  void* take(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  }
};

// Y = act(X W^T + b) + residual for any row count.  Up to 128 rows the weight-streaming kernel is the
// faster one (measured with weights that do not sit in the last-level cache: 156 / 204 us against
// 163 / 212 us for the four OPT-13B GEMMs at 32 / 128 rows); from there on the MFMA tile kernel,
// split over K where its tiles alone would not fill the chip (287 against 364 us at 256 rows).
// Decode-sized calls (<= 256 rows) are timed as their own class whichever kernel runs.
constexpr int kStreamMaxRows = 128;
constexpr int kRowPad = 64;  // elements of padding per row of a padded internal buffer (128 bytes)
bool use_skinny(int rows, int in_f) { return rows <= kStreamMaxRows && in_f % 128 == 0; }

ds_status linear(ds_ctx* ctx, const void* x, const void* w, int rows, int in_f, int out_f,
                 const ds::Epilogue& ep, void* gemm_ws, hipStream_t stream,
                 const ds::SkinnyFused* fused = nullptr, bool* fused_done = nullptr) {
  if (fused_done) *fused_done = false;
  hipError_t e;
  {
    Timed t(ctx, stream, rows <= kSkinnyMaxRows ? DS_K_SKINNY_GEMM : DS_K_GEMM);
    if (use_skinny(rows, in_f))
      e = ds::launch_skinny_gemm(x, w, rows, out_f, in_f, ep, gemm_ws, stream, fused, fused_done);
    else
      e = ds::launch_gemm(x, w, rows, out_f, in_f, ep, stream, gemm_ws, fused, fused_done);
  }
  if (e != hipSuccess) return fail(ctx, DS_ERR_HIP, "gemm failed: %s", hipGetErrorString(e));
  return DS_OK;
}

// split-K partials of the kernel that `linear` picks for exactly `rows` rows
size_t linear_ws_exact(int rows, int in_f, int out_f) {
  return use_skinny(rows, in_f) ? ds::skinny_workspace_bytes(rows, out_f, in_f)
                                : ds::gemm_workspace_bytes(rows, out_f, in_f);
}

// ... and for any row count up to `rows` (fewer rows can mean more splits), so that a workspace sized
// for a maximum serves every smaller call.  Up to 256 rows the plan may change with every row count; above,
// only with the number of row tiles (multiples of 64).
size_t linear_ws(int rows, int in_f, int out_f) {
  size_t need = 0;
  for (int r = 1; r <= rows; r = r < 256 ? r + 1 : r + 64) {
    const size_t b = linear_ws_exact(r, in_f, out_f);
    if (b > need) need = b;
  }
  const size_t b = linear_ws_exact(rows, in_f, out_f);
  return b > need ? b : need;
}

size_t max_gemm_ws(const ds_model_cfg& c, int rows) {
  size_t a = linear_ws(rows, c.hidden, qkv_width(c));
  size_t b = linear_ws(rows, c.hidden, c.hidden);
  size_t d = linear_ws(rows, c.hidden, c.ffn);
  size_t e = linear_ws(rows, c.ffn, c.hidden);
  size_t m = a > b ? a : b;
  m = m > d ? m : d;
  return m > e ? m : e;
}

// Every call that launches goes through here first: the device's one-time set-up (normally done by ds_create;
// repeated here for a context that is used on another device than it was created on).
ds_status ensure_device(ds_ctx* ctx, const DeviceState** out = nullptr) {
  hipError_t e;
  const DeviceState* st = device_state(&e);
  if (!st) return fail(ctx, DS_ERR_HIP, "device set-up failed: %s", hipGetErrorString(e));
  if (out) *out = st;
  return DS_OK;
}

// ---- debug validation of device index arrays (ctx->validate) ----
ds_status fetch_i32(ds_ctx* ctx, const int32_t* dev, size_t n, hipStream_t s, std::vector<int32_t>& out) {
  out.resize(n);
  hipError_t e = hipMemcpyAsync(out.data(), dev, n * sizeof(int32_t), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail(ctx, DS_ERR_HIP, "validation copy failed: %s", hipGetErrorString(e));
  return DS_OK;
}

// cu_seqlens [B+1]: starts at 0, ends at t, every length in [1, max_seqlen]
ds_status validate_cu(ds_ctx* ctx, const char* who, const int32_t* cu_dev, int B, int t, int max_seqlen,
                      hipStream_t s, std::vector<int32_t>& cu) {
  ds_status st = fetch_i32(ctx, cu_dev, (size_t)B + 1, s, cu);
  if (st != DS_OK) return st;
  if (cu[0] != 0) return fail(ctx, DS_ERR_BOUNDS, "%s: cu_seqlens[0] = %d, must be 0", who, cu[0]);
  for (int i = 0; i < B; ++i) {
    const long len = (long)cu[i + 1] - cu[i];
    if (len < 1) return fail(ctx, DS_ERR_BOUNDS, "%s: cu_seqlens not increasing at sequence %d", who, i);
    if (len > max_seqlen)
      return fail(ctx, DS_ERR_BOUNDS, "%s: sequence %d has %ld tokens > max_seqlen %d", who, i, len, max_seqlen);
  }
  if (cu[B] != t) return fail(ctx, DS_ERR_BOUNDS, "%s: cu_seqlens[B] = %d, must be t = %d", who, cu[B], t);
  return DS_OK;
}

// the first ceil(tokens[i] / page) entries of every row of block_tables name a block in [0, num_blocks)
ds_status validate_tables(ds_ctx* ctx, const char* who, const int32_t* bt_dev, int B, int max_blocks,
                          int num_blocks, const std::vector<int32_t>& tokens, hipStream_t s) {
  std::vector<int32_t> bt;
  ds_status st = fetch_i32(ctx, bt_dev, (size_t)B * max_blocks, s, bt);
  if (st != DS_OK) return st;
  const int page = ctx->cfg.block_size;
  for (int i = 0; i < B; ++i) {
    const long pages = ((long)tokens[i] + page - 1) / page;
    if (pages > max_blocks)
      return fail(ctx, DS_ERR_BOUNDS, "%s: sequence %d needs %ld pages > max_blocks_per_seq %d", who, i, pages,
                  max_blocks);
    for (long j = 0; j < pages; ++j) {
      const int32_t id = bt[(size_t)i * max_blocks + j];
      if (id < 0 || id >= num_blocks)
        return fail(ctx, DS_ERR_BOUNDS, "%s: block_tables[%d][%ld] = %d outside [0, %d)", who, i, j, id, num_blocks);
    }
  }
  return DS_OK;
}

// lengths [B] of a decode call: lens[i] + add in [lo, bound]; on return `tokens` holds lens[i] + add
ds_status validate_lens(ds_ctx* ctx, const char* who, const int32_t* lens_dev, int B, int add, int lo, int bound,
                        hipStream_t s, std::vector<int32_t>& tokens) {
  ds_status st = fetch_i32(ctx, lens_dev, (size_t)B, s, tokens);
  if (st != DS_OK) return st;
  for (int i = 0; i < B; ++i) {
    const long l = (long)tokens[i] + add;
    if (l < lo || l > bound)
      return fail(ctx, DS_ERR_BOUNDS, "%s: sequence %d attends over %ld tokens, outside [%d, %d]", who, i, l, lo,
                  bound);
    tokens[i] = (int32_t)l;
  }
  return DS_OK;
}

ds_status check_weights(ds_ctx* ctx, const ds_layer_weights* w) {
  if (!w) return fail(ctx, DS_ERR_INVALID_ARG, "weights is NULL");
  const void* need[] = {w->ln1_g, w->ln1_b, w->w_qkv, w->w_o, w->ln2_g, w->ln2_b, w->w_fc1, w->w_fc2};
  for (const void* p : need)
    if (!p || !aligned16(p)) return fail(ctx, DS_ERR_INVALID_ARG, "a required weight pointer is NULL or misaligned");
  const void* opt[] = {w->b_qkv, w->b_o, w->b_fc1, w->b_fc2};
  for (const void* p : opt)
    if (p && !aligned16(p)) return fail(ctx, DS_ERR_INVALID_ARG, "a bias pointer is misaligned");
  return DS_OK;
}

}  // namespace

extern "C" {

ds_status ds_create(const ds_model_cfg* cfg, ds_ctx** out) {
  if (!cfg || !out) return DS_ERR_INVALID_ARG;
  *out = nullptr;
  if (cfg->hidden <= 0 || cfg->n_heads <= 0 || cfg->head_dim <= 0 || cfg->ffn <= 0) return DS_ERR_INVALID_ARG;
  if (cfg->hidden != cfg->n_heads * cfg->head_dim) return DS_ERR_INVALID_ARG;
  const int n_kv = cfg->n_kv_heads == 0 ? cfg->n_heads : cfg->n_kv_heads;
  if (n_kv < 0 || n_kv > cfg->n_heads || cfg->n_heads % n_kv != 0) return DS_ERR_INVALID_ARG;
  if (!(cfg->ln_eps > 0.f)) return DS_ERR_INVALID_ARG;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return DS_ERR_UNSUPPORTED;
  if (cfg->block_size != 16) return DS_ERR_UNSUPPORTED;
  if (cfg->hidden % 64 != 0 || cfg->ffn % 64 != 0 || cfg->hidden > 16384) return DS_ERR_UNSUPPORTED;
  ds_ctx* c = new (std::nothrow) ds_ctx();
  if (!c) return DS_ERR_INVALID_ARG;
  c->cfg = *cfg;
  c->cfg.n_kv_heads = n_kv;
  c->err[0] = 0;
  c->profile = false;
  const char* dbg = getenv("DS_DEBUG_VALIDATE");
  c->validate = dbg && dbg[0] && strcmp(dbg, "0") != 0;
  // One-time set-up of the current device (kernel attributes, scratch address).  Without a usable device
  // the context is still good for the size queries; the first call that launches reports the failure.
  hipError_t e;
  (void)device_state(&e);
  *out = c;
  return DS_OK;
}

ds_status ds_set_validate(ds_ctx* ctx, int32_t on) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  ctx->validate = on != 0;
  return DS_OK;
}


void ds_destroy(ds_ctx* ctx) {
  if (!ctx) return;
  for (auto& r : ctx->recs) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  for (auto e : ctx->pool) (void)hipEventDestroy(e);
  delete ctx;
}

const char* ds_last_error(const ds_ctx* ctx) { return ctx ? ctx->err : "ctx is NULL"; }

size_t ds_prefill_workspace_bytes(const ds_ctx* ctx, int32_t max_tokens) {
  if (!ctx || max_tokens <= 0) return 0;
  const auto hit = ctx->prefill_ws.find(max_tokens);
  if (hit != ctx->prefill_ws.end()) return hit->second;
  const ds_model_cfg& c = ctx->cfg;
  const size_t th = align_up((size_t)max_tokens * c.hidden * 2, 256);
  const size_t tm = align_up((size_t)max_tokens * (c.ffn + kRowPad) * 2, 256);
  // a (LN out, reused for LN2), q, o, x1, u (rows padded), + split-K partials of the GEMMs
  const size_t need = 4 * th + tm + align_up(max_gemm_ws(c, max_tokens), 256);
  if (ctx->prefill_ws.size() < 4096) ctx->prefill_ws[max_tokens] = need;
  return need;
}

size_t ds_decode_workspace_bytes(const ds_ctx* ctx, int32_t max_batch, int32_t max_ctx) {
  if (!ctx || max_batch <= 0 || max_ctx <= 0) return 0;
  // the attention partials depend on max_ctx only through its page count
  const std::pair<int, int> key(max_batch, (max_ctx + 15) / 16);
  const auto hit = ctx->decode_ws.find(key);
  if (hit != ctx->decode_ws.end()) return hit->second;
  const ds_model_cfg& c = ctx->cfg;
  const size_t bh = align_up((size_t)max_batch * c.hidden * 2, 256);
  const size_t b3h = align_up((size_t)max_batch * qkv_width(c) * 2, 256);
  const size_t bm = align_up((size_t)max_batch * c.ffn * 2, 256);
  // fewer sequences can mean more splits of the KV axis: size the partials for any batch up to max_batch
  size_t att = 0;
  for (int b = 1; b <= max_batch; ++b) {
    const size_t v = ds::decode_attention_workspace_bytes(b, c.n_heads, c.n_kv_heads, c.head_dim, max_ctx);
    if (v > att) att = v;
  }
  att = align_up(att, 256);
  const size_t sk = align_up(max_gemm_ws(c, max_batch), 256);
  // a, qkv, o, x1, u, attention partials, split-K partials
  const size_t need = 3 * bh + b3h + bm + att + sk;
  if (ctx->decode_ws.size() < 4096) ctx->decode_ws[key] = need;
  return need;
}

ds_status ds_layernorm(ds_ctx* ctx, const void* x, const void* gamma, const void* beta, int32_t rows,
                       void* out, void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  if (!x || !gamma || !beta || !out || rows <= 0) return fail(ctx, DS_ERR_INVALID_ARG, "ds_layernorm: bad argument");
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(out))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_layernorm: pointers must be 16-byte aligned");
  if (ds_status st = ensure_device(ctx)) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  DS_LAUNCH(ctx, s, DS_K_LAYERNORM, ds::launch_layernorm(x, gamma, beta, out, rows, ctx->cfg.hidden, ctx->cfg.ln_eps, s));
  return DS_OK;
}

size_t ds_linear_workspace_bytes(const ds_ctx* ctx, int32_t rows, int32_t in_f, int32_t out_f) {
  if (!ctx || rows <= 0 || in_f <= 0 || out_f <= 0) return 0;
  return in_f % 64 == 0 ? linear_ws_exact(rows, in_f, out_f) : 0;
}

ds_status ds_linear_plan(const ds_ctx* ctx, int32_t rows, int32_t in_f, int32_t out_f, int32_t* streaming,
                         int32_t* tile_rows, int32_t* tile_cols, int32_t* splits, int32_t* cut_cols) {
  if (!ctx || !streaming || !tile_rows || !tile_cols || !splits || !cut_cols || rows <= 0 || in_f <= 0 ||
      out_f <= 0 || in_f % 64 != 0)
    return DS_ERR_INVALID_ARG;
  *streaming = use_skinny(rows, in_f) ? 1 : 0;
  *tile_rows = *tile_cols = *cut_cols = 0;
  *splits = 1;
  if (*streaming) {
    int tc, sp;
    ds::skinny_describe(rows, out_f, in_f, &tc, &sp);
    *tile_cols = tc; *splits = sp;
  } else {
    int tr, tc, sp, cut;
    ds::gemm_describe(rows, out_f, in_f, &tr, &tc, &sp, &cut);
    *tile_rows = tr; *tile_cols = tc; *splits = sp; *cut_cols = cut;
  }
  return DS_OK;
}

ds_status ds_linear(ds_ctx* ctx, const void* x, const void* w, const void* bias, const void* residual,
                    int32_t relu, int32_t rows, int32_t in_f, int32_t out_f, void* y, void* workspace,
                    size_t workspace_bytes, void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  if (!x || !w || !y || rows <= 0 || in_f <= 0 || out_f <= 0)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_linear: NULL pointer or non-positive size");
  if (in_f % 64 != 0 || out_f % 8 != 0)
    return fail(ctx, DS_ERR_UNSUPPORTED, "ds_linear: in_f must be a multiple of 64 and out_f of 8");
  if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(bias) || !aligned16(residual) ||
      !aligned16(workspace))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_linear: pointers must be 16-byte aligned");
  const size_t need = ds_linear_workspace_bytes(ctx, rows, in_f, out_f);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(ctx, DS_ERR_WORKSPACE, "ds_linear: workspace %zu < %zu", workspace_bytes, need);
  if (ds_status st = ensure_device(ctx)) return st;
  ds::Epilogue ep;
  ep.bias = bias;
  ep.residual = residual;
  ep.relu = relu;
  ep.out[0] = y;
  ep.seg_cols = out_f;
  return linear(ctx, x, w, rows, in_f, out_f, ep, workspace, static_cast<hipStream_t>(stream));
}

ds_status ds_embed(ds_ctx* ctx, const int32_t* token_ids, const int32_t* positions, const void* tok_emb,
                   int32_t vocab, const void* pos_emb, int32_t n_pos, int32_t rows, void* x, void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  if (!token_ids || !tok_emb || !x || rows <= 0 || vocab <= 0)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_embed: NULL pointer or non-positive size");
  if (pos_emb && (!positions || n_pos <= 0))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_embed: a position table needs positions and n_pos > 0");
  if (!aligned16(tok_emb) || !aligned16(pos_emb) || !aligned16(x))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_embed: tables and x must be 16-byte aligned");
  if (ds_status st = ensure_device(ctx)) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  DS_LAUNCH(ctx, s, DS_K_TOKEN_IO,
            ds::launch_embed(token_ids, positions, tok_emb, vocab, pos_emb, n_pos, rows, ctx->cfg.hidden, x, s));
  return DS_OK;
}

size_t ds_next_token_workspace_bytes(const ds_ctx* ctx, int32_t rows, int32_t vocab) {
  if (!ctx || rows <= 0 || rows > kSkinnyMaxRows || vocab <= 0) return 0;
  const size_t a = align_up((size_t)rows * ctx->cfg.hidden * 2, 256);
  return a + align_up(ds::skinny_argmax_workspace_bytes(rows, vocab, ctx->cfg.hidden), 256);
}

ds_status ds_next_token(ds_ctx* ctx, const void* x, const int32_t* row_index, int32_t rows, const void* ln_g,
                        const void* ln_b, const void* w_vocab, int32_t vocab, int32_t* next_token,
                        float* best_logit, void* workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  if (!x || !ln_g || !ln_b || !w_vocab || !next_token || rows <= 0 || vocab <= 0)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_next_token: NULL pointer or non-positive size");
  if (rows > kSkinnyMaxRows)
    return fail(ctx, DS_ERR_UNSUPPORTED, "ds_next_token: at most %d rows per call", kSkinnyMaxRows);
  if (vocab % 8 != 0 || ctx->cfg.hidden % 128 != 0)
    return fail(ctx, DS_ERR_UNSUPPORTED, "ds_next_token: vocab must be a multiple of 8 and hidden of 128");
  if (!aligned16(x) || !aligned16(ln_g) || !aligned16(ln_b) || !aligned16(w_vocab) || !aligned16(workspace))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_next_token: pointers must be 16-byte aligned");
  const size_t need = ds_next_token_workspace_bytes(ctx, rows, vocab);
  if (!workspace || workspace_bytes < need)
    return fail(ctx, DS_ERR_WORKSPACE, "ds_next_token: workspace %zu < %zu", workspace_bytes, need);
  if (ds_status st = ensure_device(ctx)) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  Carver cv(workspace);
  void* a = cv.take((size_t)rows * ctx->cfg.hidden * 2);
  void* cand = cv.take(ds::skinny_argmax_workspace_bytes(rows, vocab, ctx->cfg.hidden));
  DS_LAUNCH(ctx, s, DS_K_LAYERNORM,
            ds::launch_layernorm(x, ln_g, ln_b, a, rows, ctx->cfg.hidden, ctx->cfg.ln_eps, s, row_index));
  DS_LAUNCH(ctx, s, DS_K_TOKEN_IO,
            ds::launch_skinny_argmax(a, w_vocab, rows, vocab, ctx->cfg.hidden, cand, next_token, best_logit, s));
  return DS_OK;
}

ds_status ds_prefill_attention(ds_ctx* ctx, const void* q, const void* k, const void* v,
                               const int32_t* cu_seqlens, int32_t B, int32_t t, int32_t max_seqlen, void* o,
                               void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  if (!q || !k || !v || !o || !cu_seqlens || B <= 0 || t <= 0 || max_seqlen <= 0 || max_seqlen > t)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_prefill_attention: bad argument");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_prefill_attention: pointers must be 16-byte aligned");
  if (ds_status st = ensure_device(ctx)) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (ctx->validate) {
    std::vector<int32_t> cu;
    if (ds_status st = validate_cu(ctx, "ds_prefill_attention", cu_seqlens, B, t, max_seqlen, s, cu)) return st;
  }
  DS_LAUNCH(ctx, s, DS_K_PREFILL_ATTN,
            ds::launch_prefill_attention(q, k, v, cu_seqlens, B, t, max_seqlen, ctx->cfg.n_heads, ctx->cfg.n_kv_heads,
                                         ctx->cfg.head_dim, o, s));
  return DS_OK;
}

ds_status ds_prefill(ds_ctx* ctx, const ds_layer_weights* w, const void* x, const int32_t* cu_seqlens,
                     int32_t B, int32_t t, int32_t max_seqlen, void* y, void* k_out, void* v_out,
                     void* workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  ds_status st = check_weights(ctx, w);
  if (st != DS_OK) return st;
  if (!x || !cu_seqlens || !y || !k_out || !v_out)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_prefill: NULL pointer");
  if (B <= 0 || t <= 0 || max_seqlen <= 0 || max_seqlen > t || B > t)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_prefill: need B>0, t>0, 0<max_seqlen<=t, B<=t");
  if (x == y) return fail(ctx, DS_ERR_INVALID_ARG, "ds_prefill: y must not alias x");
  if (!aligned16(x) || !aligned16(y) || !aligned16(k_out) || !aligned16(v_out) || !aligned16(workspace))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_prefill: pointers must be 16-byte aligned");
  const size_t need = ds_prefill_workspace_bytes(ctx, t);
  if (!workspace || workspace_bytes < need)
    return fail(ctx, DS_ERR_WORKSPACE, "ds_prefill: workspace %zu < %zu", workspace_bytes, need);
  if ((st = ensure_device(ctx)) != DS_OK) return st;

  const ds_model_cfg& c = ctx->cfg;
  const int h = c.hidden, m = c.ffn;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (ctx->validate) {
    std::vector<int32_t> cu;
    if ((st = validate_cu(ctx, "ds_prefill", cu_seqlens, B, t, max_seqlen, s, cu)) != DS_OK) return st;
  }
  Carver ws(workspace);
  void* a = ws.take((size_t)t * h * 2);
  void* q = ws.take((size_t)t * h * 2);
  void* o = ws.take((size_t)t * h * 2);
  void* x1 = ws.take((size_t)t * h * 2);
  // The FFN intermediate is written by one tile GEMM and read by the next: give its rows 128 bytes of
  // padding so that consecutive rows do not start on the same memory channels (m * 2 bytes is a multiple of
  // 8 KB for every OPT size; at OPT-175B's 96 KB the dense stride costs the second GEMM a quarter of its rate).
  const bool pad_u = !use_skinny(t, h) && !use_skinny(t, m) && ds::gemm_splits(t, m, h) == 1 &&
                     ds::gemm_splits(t, h, m) == 1;
  const int ld_u = pad_u ? m + kRowPad : m;
  void* u = ws.take((size_t)t * (m + kRowPad) * 2);
  void* sk = ws.take(0);

  // a = LN1(x)
  DS_LAUNCH(ctx, s, DS_K_LAYERNORM, ds::launch_layernorm(x, w->ln1_g, w->ln1_b, a, t, h, c.ln_eps, s));
  // [q | k_out | v_out] = a W_qkv^T + b_qkv
  {
    ds::Epilogue ep;
    ep.bias = w->b_qkv;
    ep.out[0] = q; ep.out[1] = k_out; ep.out[2] = v_out;
    ep.seg_cols = h;
    ep.seg_cols_kv = kv_width(c);
    st = linear(ctx, a, w->w_qkv, t, h, qkv_width(c), ep, sk, s);
    if (st != DS_OK) return st;
  }
  // o = causal attention per request
  DS_LAUNCH(ctx, s, DS_K_PREFILL_ATTN,
            ds::launch_prefill_attention(q, k_out, v_out, cu_seqlens, B, t, max_seqlen, c.n_heads, c.n_kv_heads,
                                         c.head_dim, o, s));
  // x1 = x + o W_o^T + b_o
  {
    ds::Epilogue ep;
    ep.bias = w->b_o; ep.residual = x;
    ep.out[0] = x1; ep.seg_cols = h;
    st = linear(ctx, o, w->w_o, t, h, h, ep, sk, s);
    if (st != DS_OK) return st;
  }
  // f = LN2(x1) (reuses a)
  DS_LAUNCH(ctx, s, DS_K_LAYERNORM, ds::launch_layernorm(x1, w->ln2_g, w->ln2_b, a, t, h, c.ln_eps, s));
  // u = relu(f W_1^T + b_1)
  {
    ds::Epilogue ep;
    ep.bias = w->b_fc1; ep.relu = 1;
    ep.out[0] = u; ep.seg_cols = m;
    if (pad_u) ep.out_ld = ld_u;
    st = linear(ctx, a, w->w_fc1, t, h, m, ep, sk, s);
    if (st != DS_OK) return st;
  }
  // y = x1 + u W_2^T + b_2
  {
    ds::Epilogue ep;
    ep.bias = w->b_fc2; ep.residual = x1;
    ep.out[0] = y; ep.seg_cols = h;
    if (pad_u) ep.x_ld = ld_u;
    st = linear(ctx, u, w->w_fc2, t, m, h, ep, sk, s);
    if (st != DS_OK) return st;
  }
  return DS_OK;
}

ds_status ds_kv_migrate(ds_ctx* ctx, const void* k_src, const void* v_src, const int32_t* cu_seqlens,
                        int32_t B, int32_t t, int32_t max_seqlen, const int32_t* block_tables,
                        int32_t max_blocks_per_seq, void* k_cache, void* v_cache, int32_t num_blocks,
                        void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  if (!k_src || !v_src || !cu_seqlens || !block_tables || !k_cache || !v_cache)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_kv_migrate: NULL pointer");
  if (B <= 0 || t <= 0 || max_seqlen <= 0 || max_seqlen > t || num_blocks <= 0 || max_blocks_per_seq <= 0)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_kv_migrate: non-positive or inconsistent size");
  if ((int64_t)max_blocks_per_seq * ctx->cfg.block_size < max_seqlen)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_kv_migrate: max_seqlen %d does not fit %d blocks per sequence",
                max_seqlen, max_blocks_per_seq);
  if (!aligned16(k_src) || !aligned16(v_src) || !aligned16(k_cache) || !aligned16(v_cache))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_kv_migrate: pointers must be 16-byte aligned");
  if (ds_status st = ensure_device(ctx)) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (ctx->validate) {
    std::vector<int32_t> cu, lens((size_t)B);
    if (ds_status st = validate_cu(ctx, "ds_kv_migrate", cu_seqlens, B, t, max_seqlen, s, cu)) return st;
    for (int i = 0; i < B; ++i) lens[i] = cu[i + 1] - cu[i];
    if (ds_status st = validate_tables(ctx, "ds_kv_migrate", block_tables, B, max_blocks_per_seq, num_blocks, lens, s))
      return st;
  }
  DS_LAUNCH(ctx, s, DS_K_KV_MIGRATE,
            ds::launch_kv_migrate(k_src, v_src, cu_seqlens, B, max_seqlen, block_tables, max_blocks_per_seq,
                                  k_cache, v_cache, ctx->cfg.n_kv_heads, ctx->cfg.head_dim, s));
  return DS_OK;
}

ds_status ds_decode_attention(ds_ctx* ctx, const void* q, const int32_t* kv_lens, const int32_t* block_tables,
                              int32_t B, int32_t max_blocks_per_seq, int32_t max_kv_len, const void* k_cache,
                              const void* v_cache, int32_t num_blocks, void* o, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  if (!q || !kv_lens || !block_tables || !k_cache || !v_cache || !o)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_decode_attention: NULL pointer");
  if (B <= 0 || max_kv_len <= 0 || num_blocks <= 0 || max_blocks_per_seq <= 0 ||
      (int64_t)max_blocks_per_seq * ctx->cfg.block_size < max_kv_len)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_decode_attention: non-positive or inconsistent size");
  if (!aligned16(q) || !aligned16(o) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(workspace))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_decode_attention: pointers must be 16-byte aligned");
  const ds_model_cfg& c = ctx->cfg;
  const size_t need = ds::decode_attention_workspace_bytes(B, c.n_heads, c.n_kv_heads, c.head_dim, max_kv_len);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(ctx, DS_ERR_WORKSPACE, "ds_decode_attention: workspace %zu < %zu", workspace_bytes, need);
  if (ds_status st = ensure_device(ctx)) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (ctx->validate) {
    std::vector<int32_t> lens;
    if (ds_status st = validate_lens(ctx, "ds_decode_attention", kv_lens, B, 0, 0, max_kv_len, s, lens)) return st;
    if (ds_status st = validate_tables(ctx, "ds_decode_attention", block_tables, B, max_blocks_per_seq, num_blocks,
                                       lens, s))
      return st;
  }
  DS_LAUNCH(ctx, s, DS_K_DECODE_ATTN,
            ds::launch_decode_attention(q, c.hidden, kv_lens, 0, block_tables, B, max_blocks_per_seq, max_kv_len,
                                        k_cache, v_cache, c.n_heads, c.n_kv_heads, c.head_dim, o, workspace, s));
  return DS_OK;
}

// Both decode-step entry points: `workspace` is the caller's buffer, or null for the static scratch array
// of the current device (then the step must fit DS_STATIC_SCRATCH_BYTES).
static ds_status decode_step(ds_ctx* ctx, const ds_layer_weights* w, const void* x, const int32_t* ctx_lens,
                             const int32_t* block_tables, int32_t B, int32_t max_blocks_per_seq, int32_t max_ctx,
                             void* k_cache, void* v_cache, int32_t num_blocks, void* y, void* workspace,
                             size_t workspace_bytes, bool use_static, void* stream) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  ds_status st = check_weights(ctx, w);
  if (st != DS_OK) return st;
  if (!x || !ctx_lens || !block_tables || !k_cache || !v_cache || !y)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_decode_step: NULL pointer");
  if (B <= 0 || max_ctx <= 0 || num_blocks <= 0 || max_blocks_per_seq <= 0)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_decode_step: non-positive size");
  if ((int64_t)max_blocks_per_seq * ctx->cfg.block_size < max_ctx)
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_decode_step: max_ctx %d does not fit %d blocks per sequence", max_ctx,
                max_blocks_per_seq);
  if (x == y) return fail(ctx, DS_ERR_INVALID_ARG, "ds_decode_step: y must not alias x");
  if (!aligned16(x) || !aligned16(y) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(workspace))
    return fail(ctx, DS_ERR_INVALID_ARG, "ds_decode_step: pointers must be 16-byte aligned");
  const size_t need = ds_decode_workspace_bytes(ctx, B, max_ctx);
  const DeviceState* dev = nullptr;
  if (use_static) {
    if (need > (size_t)DS_STATIC_SCRATCH_BYTES)
      return fail(ctx, DS_ERR_WORKSPACE,
                  "ds_decode_step_static: this step needs %zu bytes of scratch, the static array holds %zu "
                  "(use ds_decode_step with a workspace)", need, (size_t)DS_STATIC_SCRATCH_BYTES);
    if ((st = ensure_device(ctx, &dev)) != DS_OK) return st;
    workspace = dev->scratch;
    workspace_bytes = (size_t)DS_STATIC_SCRATCH_BYTES;
  } else {
    if (!workspace || workspace_bytes < need)
      return fail(ctx, DS_ERR_WORKSPACE, "ds_decode_step: workspace %zu < %zu", workspace_bytes, need);
    if ((st = ensure_device(ctx)) != DS_OK) return st;
  }

  const ds_model_cfg& c = ctx->cfg;
  const int h = c.hidden, m = c.ffn;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (ctx->validate) {
    std::vector<int32_t> lens;
    if ((st = validate_lens(ctx, "ds_decode_step", ctx_lens, B, 1, 1, max_ctx, s, lens)) != DS_OK) return st;
    if ((st = validate_tables(ctx, "ds_decode_step", block_tables, B, max_blocks_per_seq, num_blocks, lens, s)) !=
        DS_OK)
      return st;
  }
  Carver ws(workspace);
  void* a = ws.take((size_t)B * h * 2);
  void* o = ws.take((size_t)B * h * 2);
  void* x1 = ws.take((size_t)B * h * 2);
  const int hkv = kv_width(c), wqkv = qkv_width(c);
  void* qkv = ws.take((size_t)B * wqkv * 2);
  void* u = ws.take((size_t)B * m * 2);
  void* att = ws.take(ds::decode_attention_workspace_bytes(B, c.n_heads, c.n_kv_heads, c.head_dim, max_ctx));
  void* sk = ws.take(0);

  DS_LAUNCH(ctx, s, DS_K_LAYERNORM, ds::launch_layernorm(x, w->ln1_g, w->ln1_b, a, B, h, c.ln_eps, s));
  const uint16_t* qkv16 = static_cast<const uint16_t*>(qkv);
  {
    // [q | k | v] = a W_qkv^T + b_qkv; the split-K reduction writes k, v straight into the cache
    ds::Epilogue ep;
    ep.bias = w->b_qkv;
    ep.out[0] = qkv; ep.seg_cols = wqkv;
    ds::SkinnyFused fu;
    fu.kind = ds::SkinnyFused::kKvAppend;
    fu.ctx_lens = ctx_lens; fu.block_tables = block_tables; fu.max_blocks = max_blocks_per_seq;
    fu.k_cache = k_cache; fu.v_cache = v_cache;
    fu.n_heads = c.n_heads; fu.n_kv_heads = c.n_kv_heads; fu.head_dim = c.head_dim;
    bool appended = false;
    st = linear(ctx, a, w->w_qkv, B, h, wqkv, ep, sk, s, &fu, &appended);
    if (st != DS_OK) return st;
    if (!appended)
      DS_LAUNCH(ctx, s, DS_K_KV_APPEND,
                ds::launch_kv_append(qkv16 + h, qkv16 + h + hkv, wqkv, ctx_lens, block_tables, B, max_blocks_per_seq,
                                     k_cache, v_cache, c.n_kv_heads, c.head_dim, s));
  }
  DS_LAUNCH(ctx, s, DS_K_DECODE_ATTN,
            ds::launch_decode_attention(qkv, wqkv, ctx_lens, 1, block_tables, B, max_blocks_per_seq, max_ctx,
                                        k_cache, v_cache, c.n_heads, c.n_kv_heads, c.head_dim, o, att, s));
  {
    // x1 = x + o W_o^T + b_o, and f = LN2(x1) in the same reduction pass
    ds::Epilogue ep;
    ep.bias = w->b_o; ep.residual = x;
    ep.out[0] = x1; ep.seg_cols = h;
    ds::SkinnyFused fu;
    fu.kind = ds::SkinnyFused::kLayerNorm;
    fu.ln_gamma = w->ln2_g; fu.ln_beta = w->ln2_b; fu.ln_eps = c.ln_eps; fu.ln_out = a;
    bool normed = false;
    st = linear(ctx, o, w->w_o, B, h, h, ep, sk, s, &fu, &normed);
    if (st != DS_OK) return st;
    if (!normed)
      DS_LAUNCH(ctx, s, DS_K_LAYERNORM, ds::launch_layernorm(x1, w->ln2_g, w->ln2_b, a, B, h, c.ln_eps, s));
  }
  {
    ds::Epilogue ep;
    ep.bias = w->b_fc1; ep.relu = 1;
    ep.out[0] = u; ep.seg_cols = m;
    st = linear(ctx, a, w->w_fc1, B, h, m, ep, sk, s);
    if (st != DS_OK) return st;
  }
  {
    ds::Epilogue ep;
    ep.bias = w->b_fc2; ep.residual = x1;
    ep.out[0] = y; ep.seg_cols = h;
    st = linear(ctx, u, w->w_fc2, B, m, h, ep, sk, s);
    if (st != DS_OK) return st;
  }
  return DS_OK;
}

ds_status ds_decode_step(ds_ctx* ctx, const ds_layer_weights* w, const void* x, const int32_t* ctx_lens,
                         const int32_t* block_tables, int32_t B, int32_t max_blocks_per_seq, int32_t max_ctx,
                         void* k_cache, void* v_cache, int32_t num_blocks, void* y, void* workspace,
                         size_t workspace_bytes, void* stream) {
  return decode_step(ctx, w, x, ctx_lens, block_tables, B, max_blocks_per_seq, max_ctx, k_cache, v_cache,
                     num_blocks, y, workspace, workspace_bytes, false, stream);
}

ds_status ds_decode_step_static(ds_ctx* ctx, const ds_layer_weights* w, const void* x, const int32_t* ctx_lens,
                                const int32_t* block_tables, int32_t B, int32_t max_blocks_per_seq,
                                int32_t max_ctx, void* k_cache, void* v_cache, int32_t num_blocks, void* y,
                                void* stream) {
  return decode_step(ctx, w, x, ctx_lens, block_tables, B, max_blocks_per_seq, max_ctx, k_cache, v_cache,
                     num_blocks, y, nullptr, 0, true, stream);
}

ds_status ds_profile_enable(ds_ctx* ctx, int32_t on) {
  if (!ctx) return DS_ERR_INVALID_ARG;
  ctx->profile = on != 0;
  return DS_OK;
}

ds_status ds_profile_collect(ds_ctx* ctx, double* ms, int64_t* launches) {
  if (!ctx || !ms || !launches) return DS_ERR_INVALID_ARG;
  for (int i = 0; i < DS_K_COUNT; ++i) {
    ms[i] = 0.0;
    launches[i] = 0;
  }
  // The record is taken over first, so every event goes back to the pool exactly once whether or not a
  // timing call fails on the way.
  std::vector<ds_ctx::Rec> recs;
  recs.swap(ctx->recs);
  hipError_t first_err = hipSuccess;
  for (auto& r : recs) {
    float t = 0.f;
    hipError_t e = first_err;
    if (e == hipSuccess) e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.a, r.b);
    if (e != hipSuccess) {
      if (first_err == hipSuccess) first_err = e;
    } else if (r.kind >= 0 && r.kind < DS_K_COUNT) {
      ms[r.kind] += t;
      launches[r.kind] += 1;
    }
    ctx->pool.push_back(r.a);
    ctx->pool.push_back(r.b);
  }
  if (first_err != hipSuccess)
    return fail(ctx, DS_ERR_HIP, "event timing failed: %s", hipGetErrorString(first_err));
  return DS_OK;
}

}  // extern "C"
