// bf16 GEMM on the CDNA4 matrix cores for the prefill phase (and for decoding batches too wide for
// the streaming kernels):
//   Y[M,N] = act(X[M,K] W[N,K]^T + bias) + residual,  fp32 accumulate.
// Both operands are K-contiguous, so a lane's 8-element MFMA fragment is one
// 16-byte LDS read.  The tile is computed transposed (weight rows as the MFMA
// row operand, activation rows as the column operand).
//
// Tile BM x BN (activation rows x weight rows: 256x160, 256x256, 128x128 or 64x128), BK = 64,
// 256 threads = 4 waves (one per SIMD).  Operands go global -> LDS directly (no register
// staging), three LDS buffers (two for the 256x256 tile), one barrier per k-tile; fragment reads and load issue are
// interleaved with the MFMAs by hand (scheduling fences); the epilogue is
// staged through LDS so bias / residual / output move as 16-byte row pieces.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kBK = 64;

// LDS a workgroup asks for: its ring of operand stages - or the whole 160 KB of the compute unit once the ring
// alone is more than half of it (a second workgroup could not move in anyway), which gives the epilogue a
// larger staging area: more columns per pass, longer contiguous row pieces in the output stores.
constexpr int gemm_lds_bytes(int BM, int BN, int STAGES) {
  const int ring = STAGES * (BM + BN) * kBK * 2;
  return ring > 80 * 1024 ? 160 * 1024 : ring;
}

struct GemmParams {
  const uint16_t* X;
  const uint16_t* W;
  const uint16_t* bias;
  const uint16_t* residual;
  uint16_t* out[3];
  int seg_cols, seg_cols_kv;  // widths of the first and of the other two output segments
  int M, N, K;
  int relu;
  int tiles_m, tiles_n;
  int ldx;     // row stride of X in elements (>= K)
  int ld_out;  // row stride of out[0]
  int ld_res;  // row stride of residual
  int n_base;  // first output column of this launch (a launch may cover the columns [n_base, N) only)
  // Split-K (gridDim.y = S > 1): split s multiplies k-tiles s, s + S, ... and stores its fp32
  // accumulators to partial[s][M][N]; the epilogue then belongs to whoever adds the partials.
  float* partial;
  // Decode QKV projection (N = (n_heads + 2 n_kv_heads) head_dim): with k_cache set, the K and V parts of
  // row m go to slot ctx_lens[m] of the paged cache [num_blocks, n_kv_heads, 16, head_dim] instead of `out`.
  const int32_t* ctx_lens;
  const int32_t* block_tables;
  int max_blocks;
  uint16_t* k_cache;
  uint16_t* v_cache;
  int n_heads, n_kv_heads, head_dim;
#ifdef DS_DEV_SWITCHES
  unsigned long long* dbg;  // timing harness builds only: 4 wall-clock stamps per workgroup
#endif
};

#ifdef DS_DEV_SWITCHES
unsigned long long* g_gemm_dbg = nullptr;
#define DS_STAMP(i)                                                                         \
  do {                                                                                      \
    if (p.dbg && threadIdx.x == 0) p.dbg[(size_t)(blockIdx.x + gridDim.x * blockIdx.y) * 4 + (i)] = __builtin_amdgcn_s_memrealtime(); \
  } while (0)
#else
#define DS_STAMP(i)
#endif

// Tile order.  Workgroup ids are dealt round-robin to the 8 XCDs (each with a private L2).  With one
// contiguous m-fastest range of tiles per XCD and many row tiles (long prefill batches), the 32 workgroups an
// XCD runs at a time share one weight tile and read 32 different activation tiles, and the eight XCDs sit in
// far-apart parts of the output, so every column tile re-streams the whole activation matrix from HBM.
// Instead, the 256 workgroups that run together (32 per XCD, ids dealt round-robin) take one patch of up to
// 16 x 16 output tiles, and inside it every XCD a 16 x 2 strip: 16 + 16 operand tiles from HBM per 256
// output tiles, 16 + 2 through each L2 per 32.
__device__ __forceinline__ void patch_tile(int pid, int tiles_m, int tiles_n, int& tm, int& tn) {
  constexpr int kXcd = 8, kPerXcd = 32, kChunk = kXcd * kPerXcd, kGroupM = 16;
  const int total = tiles_m * tiles_n;
  const int full = total / kChunk * kChunk;
  int v = pid;
  if (pid < full) {
    const int xcd = pid % kXcd, slot = pid / kXcd;
    v = slot / kPerXcd * kChunk + xcd * kPerXcd + slot % kPerXcd;
  } else {
    const int per = (total - full) / kXcd, q = pid - full;  // last, partial chunk: equal contiguous shares
    if (q < per * kXcd) v = full + (q % kXcd) * per + q / kXcd;
  }
  const int per_group = kGroupM * tiles_n;
  const int g = v / per_group;
  const int gsz = min(kGroupM, tiles_m - g * kGroupM);
  const int r = v - g * per_group;
  tm = g * kGroupM + r % gsz;
  tn = r / gsz;
}

// ---------------------------------------------------------------------------
// Direct global->LDS loads (no register staging, no ds_write):
// each wave-level load instruction drops 64 x 16 bytes = 8 rows x 128 bytes
// into a contiguous 1 KB of LDS.  Rows are unpadded; bank conflicts are
// avoided by an XOR swizzle applied on the *global* side: LDS row r holds
// 16-byte chunk c at position c ^ ((r >> 1) & 7).  Rows are 128 bytes = half
// of the 64 banks, so even/odd rows use different halves and any 16
// consecutive rows read at the same chunk index cover all 64 banks once.  STAGES LDS buffers; the load of k-tile
// kt+STAGES-1 is in flight while k-tile kt is multiplied.
// ---------------------------------------------------------------------------
template <int VM>
__device__ __forceinline__ void wait_vmcnt() {
  // s_waitcnt with only vmcnt set: vmcnt[3:0] | expcnt=7 | lgkmcnt=15 | vmcnt[5:4] in bits 15:14
  __builtin_amdgcn_s_waitcnt((VM & 0xf) | (0x7 << 4) | (0xf << 8) | ((VM >> 4) << 14));
}

// EPI selects the epilogue at compile time, so the plain prefill instantiation carries none of the
// decode-side code: 0 = bias / ReLU / residual -> bf16 segments; 1 = split-K, raw fp32 partials;
// 2 = as 0, but the K and V thirds go into the paged cache.
enum { kEpiPlain = 0, kEpiPartial = 1, kEpiKvScatter = 2 };

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int EPI>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_dl_kernel(const GemmParams p) {
  // One wave per SIMD.  (Eight waves - two per SIMD, 128 accumulator registers each - were measured on the
  // 256x256 tile: equal as 4x2 waves of 64x128, 7 % slower as 2x4 of 128x64; the loop is not latency-bound.)
  constexpr int NW = WAVES_M * WAVES_N;
  static_assert(NW == 4, "4 waves");
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "a wave-level load covers 8 rows");
  constexpr int ROW_BYTES = kBK * 2;                      // 128
  constexpr int STAGE_ELEMS = (BM + BN) * kBK;            // elements per stage
  constexpr int XL = BM / (8 * NW);                       // X loads per wave per stage
  constexpr int WL = BN / (8 * NW);                       // W loads per wave per stage
  constexpr int LPS = XL + WL;
  static_assert((STAGES - 1) * LPS < 64, "vmcnt range");

  extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  DS_STAMP(0);
  int tile_m, tile_n;
  patch_tile(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM;
  const int n0 = p.n_base + tile_n * BN;
  const int K = p.K;
  // Split-K deals the k-tiles round-robin (split s takes tiles s, s + S, ...), as the weight-streaming
  // kernel does: the splits of one output tile read neighbouring 128-byte pieces of the same rows at
  // about the same time.  (Measured no different from contiguous K ranges per split.)
  const int kt_step = EPI == kEpiPartial ? (int)gridDim.y : 1;
  const int kt_first = EPI == kEpiPartial ? (int)blockIdx.y : 0;
  const int KT = (K / kBK - kt_first + kt_step - 1) / kt_step;  // >= 1: splits <= K / 64

  // per-lane source offsets (bytes, from the tile's first row) of this wave's loads; load j covers rows
  // 8*(NW*j+wave) .. +7.  With the tile origin and the k position in a scalar base, the lane part is a 32-bit
  // value that never changes, and a load needs no vector arithmetic at all.
  const int lrow = lane >> 3;
  const int lchunk = (lane & 7) ^ (4 * (wave & 1) + (lane >> 4));  // key = (row >> 1) & 7, row = 8*(NW*j+wave) + lane/8
  const char* xbase = reinterpret_cast<const char*>(p.X + (size_t)m0 * p.ldx);
  const char* wbase = reinterpret_cast<const char*>(p.W + (size_t)n0 * K);
  uint32_t xoff[XL], woff[WL];
#pragma unroll
  for (int j = 0; j < XL; ++j) {
    const int row = min(8 * (NW * j + wave) + lrow, p.M - 1 - m0);
    xoff[j] = ((uint32_t)row * (uint32_t)p.ldx + lchunk * 8) * 2u;
  }
#pragma unroll
  for (int j = 0; j < WL; ++j) {
    const int row = min(8 * (NW * j + wave) + lrow, p.N - 1 - n0);
    woff[j] = ((uint32_t)row * (uint32_t)K + lchunk * 8) * 2u;
  }
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);  // keep LDS destinations in scalar registers
  // Loads k-tile `kt_load` into buffer `stage`.  Tiles past the end are clamped to the last one (a
  // harmless re-load into a buffer nobody reads again): this keeps the main loop free of branches, so
  // the loads can be interleaved with MFMAs by the scheduler.
  auto issue_one = [&](int stage, int kt_load, int j) {   // j in [0, LPS): X loads first, then W loads
    const size_t kofs = (size_t)((kt_first + min(kt_load, KT - 1) * kt_step) * kBK) * 2;   // bytes
    uint16_t* xb = lds + stage * STAGE_ELEMS + wave_s * 512;     // 512 elements = 1 KB per wave-load
    // (the empty asm keeps the 32-bit lane offset a value of this basic block: hoisted out of the loop as a
    // 64-bit pair it costs a 64-bit vector add per load instead of riding in the instruction's offset operand)
    uint32_t& off = j < XL ? xoff[j < XL ? j : 0] : woff[j < XL ? 0 : j - XL];
    asm volatile("" : "+v"(off));
    if (j < XL) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xbase + kofs + off),
                                       (__attribute__((address_space(3))) void*)(xb + j * NW * 512), 16, 0, 0);
    } else {
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(wbase + kofs + off),
          (__attribute__((address_space(3))) void*)(xb + BM * kBK + (j - XL) * NW * 512), 16, 0, 0);
    }
  };
  auto issue = [&](int stage, int kt_load) {
#pragma unroll
    for (int j = 0; j < LPS; ++j) issue_one(stage, kt_load, j);
  };

  floatx16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  // swizzled fragment offsets (elements) inside a row, one per k-step
  const int frag_row = lane & 31;
  const int hl = lane >> 5;
  // Kept in registers across the k loop, one per k-step and operand (the empty asm stops the compiler from
  // recomputing them in the loop): a fragment read is then one add of the stage's base plus an immediate.
  int xfrag[kBK / 16], wfrag[kBK / 16];
#pragma unroll
  for (int kk = 0; kk < kBK / 16; ++kk) {
    const int koff = ((2 * kk + hl) ^ ((lane >> 1) & 7)) * 8;
    xfrag[kk] = (wm * WTM + frag_row) * kBK + koff;
    wfrag[kk] = BM * kBK + (wn * WTN + frag_row) * kBK + koff;
    asm volatile("" : "+v"(xfrag[kk]), "+v"(wfrag[kk]));
  }

  // A k-tile (4 MFMA k-steps) is multiplied in two halves of two k-steps each.  Within a half every
  // accumulator tile gets its two MFMAs back to back (the second one chains on the first one's
  // result, which the matrix pipe issues without a bubble; a round-robin over 10 accumulators was
  // measured ~15 % slower with one wave per SIMD).  The fragments of the next half are fetched
  // while the current half is multiplied, so two fragment sets of 2 x (TN + TM) registers exist.
  // (held as integer vectors: bf16 vectors carried around the loop get re-packed by the compiler)
  struct Frags {
    u32x4 w[2][TN];
    u32x4 x[2][TM];
  };
  Frags fa, fb;
  constexpr int NR = 2 * (TN + TM);  // fragment reads per half
  // read number r of the half starting at k-step kk0 of stage buffer sb
  auto frag_read = [&](Frags& f, const uint16_t* sb, int kk0, int r) {
    const int s2 = r / (TN + TM), q = r % (TN + TM);
    if (q < TN) f.w[s2][q] = *reinterpret_cast<const u32x4*>(sb + wfrag[kk0 + s2] + q * 32 * kBK);
    else f.x[s2][q - TN] = *reinterpret_cast<const u32x4*>(sb + xfrag[kk0 + s2] + (q - TN) * 32 * kBK);
  };

  // One half: after each accumulator's MFMA pair the code issues a share of the next half's fragment
  // reads and (in the second half of a tile) of the global->LDS loads of tile kt+3; a scheduling
  // fence after every group keeps that interleaving, so memory instructions issue in the shadow of
  // the MFMAs instead of in bursts.
  // `mem(j)` is called for j = 0 .. JN-1, spread evenly over the MFMA pairs: it issues the j-th
  // direct-to-LDS load of this half.
  auto half = [&](auto jn, const Frags& fc, Frags& fn, const uint16_t* sb_next, int kk_next, auto&& mem) {
    constexpr int NM = TM * TN;
    constexpr int JN = decltype(jn)::value;
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      const int a = i / TM, b = i % TM;
      acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fc.w[0][a]),
                                                          __builtin_bit_cast(bf16x8, fc.x[0][b]), acc[a][b], 0, 0, 0);
      acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fc.w[1][a]),
                                                          __builtin_bit_cast(bf16x8, fc.x[1][b]), acc[a][b], 0, 0, 0);
#pragma unroll
      for (int r = i * NR / NM; r < (i + 1) * NR / NM; ++r) frag_read(fn, sb_next, kk_next, r);
#pragma unroll
      for (int j = i * JN / NM; j < (i + 1) * JN / NM; ++j) mem(j);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  using none = std::integral_constant<int, 0>;
  using all_loads = std::integral_constant<int, LPS>;
  auto no_mem = [](int) {};

  // ---- epilogue set-up (used after the k-loop; the first pass's loads are issued inside it) ----
  // Each wave stages its own WTM x (GA*32) fp32 block (GA column tiles per pass) in LDS that the
  // k-loop no longer needs; rows are padded by 4 floats so the 16-byte transposing writes of 16
  // lanes fall into distinct banks.
  constexpr int LDS_FLOATS = gemm_lds_bytes(BM, BN, STAGES) / 4;
  constexpr int GA_FIT = (LDS_FLOATS / (NW * WTM) - 4) / 32;
  constexpr int GA = GA_FIT < TN ? GA_FIT : TN;
  static_assert(GA >= 1, "no room to stage the epilogue");
  constexpr int RSTR = GA * 32 + 4;  // staging row stride in floats
  constexpr int MAX_ITERS = WTM * GA * 4 / 64;
  constexpr int NPASS = (TN + GA - 1) / GA;
  const int row_base = m0 + wm * WTM;
  const int col_base = n0 + wn * WTN;
  // Pass `a0/GA` covers column tiles a0 .. a0+ga-1; after the LDS transposition lane `idx = it*64+lane`
  // owns row idx / cpr, 8-column chunk idx % cpr (cpr = 4*ga chunks per row).
  u32x4 epi_res[2][MAX_ITERS], epi_bias[2][MAX_ITERS];
  auto epi_prefetch = [&](int a0, u32x4* resv, u32x4* biasv) {
    const int ga = (TN - a0) < GA ? (TN - a0) : GA;
    const int cpr = ga * 4;
    const int iters = WTM * cpr / 64;
#pragma unroll
    for (int it = 0; it < MAX_ITERS; ++it) {
      if (it >= iters) break;
      const int idx = it * 64 + lane;
      const int r = idx / cpr, ch = idx - r * cpr;
      const int row = row_base + r, n = col_base + a0 * 32 + ch * 8;
      const bool ok = row < p.M && n < p.N;
      resv[it] = u32x4{0, 0, 0, 0};
      biasv[it] = u32x4{0, 0, 0, 0};
      if (EPI == kEpiPartial) continue;
      if (ok && p.residual) resv[it] = ld16(p.residual + (size_t)row * p.ld_res + n);
      // when cpr divides 64 the chunk (hence the bias piece) is the same for every `it`
      if (ok && p.bias && (it == 0 || 64 % cpr != 0)) biasv[it] = ld16(p.bias + n);
    }
  };

  {
    // Direct-to-LDS schedule (3 LDS buffers, ONE barrier per k-tile, two k-tiles of flight time):
    //   (written for STAGES = 3; see below for 2)
    //   iteration kt:  first half of tile kt (fetching the fragments of its second half)
    //                  wait until this wave's part of tile kt+1 has landed (tile kt+2 may still fly)
    //                  barrier: tile kt+1 is visible to all, and nobody reads buffer kt%3 any more
    //                           (the second half's fragments are already in registers)
    //                  second half of tile kt, issuing the loads of tile kt+3 into buffer kt%3 and
    //                  fetching the first-half fragments of tile kt+1
    // With two buffers the same schedule holds with one k-tile of flight time: at the barrier tile
    // kt+1 (requested during the second half of tile kt-1) must have landed completely.
    static_assert(STAGES == 2 || STAGES == 3, "ring of 2 or 3 buffers");
#pragma unroll
    for (int st = 0; st < STAGES; ++st) issue(st, st);
    wait_vmcnt<(STAGES - 1) * LPS>();
    __syncthreads();
    DS_STAMP(1);
#pragma unroll
    for (int r = 0; r < NR; ++r) frag_read(fa, lds, 0, r);

    int stage = 0;  // buffer of tile kt
    for (int kt = 0; kt < KT - 1; ++kt) {
      const uint16_t* sb = lds + stage * STAGE_ELEMS;
      int nstage = stage + 1;
      if (nstage == STAGES) nstage = 0;
      const uint16_t* sbn = lds + nstage * STAGE_ELEMS;
      __builtin_amdgcn_sched_barrier(0);
      half(none{}, fa, fb, sb, 2, no_mem);
      wait_vmcnt<(STAGES - 2) * LPS>();
      __syncthreads();
      half(all_loads{}, fb, fa, sbn, 0, [&](int j) { issue_one(stage, kt + STAGES, j); });
      stage = nstage;
    }
    // Last k-tile (already in LDS and visible since the previous iteration's barrier): no loads, no
    // waits.  The residual and bias pieces of the first epilogue pass are requested before it, so
    // their memory latency passes while the matrix pipe still has work.
    // (only where the register file has room for them next to the accumulators and both fragment sets)
    constexpr bool EARLY_EPI = TM * TN <= 10;
    if (EARLY_EPI) epi_prefetch(0, epi_res[0], epi_bias[0]);
    {
      const uint16_t* sb = lds + stage * STAGE_ELEMS;
      __builtin_amdgcn_sched_barrier(0);
      half(none{}, fa, fb, sb, 2, no_mem);
      // (the fragment fetch of this half reads a buffer of clamped re-loads; the values are never used)
      half(none{}, fb, fa, sb, 0, no_mem);
    }
    if (!EARLY_EPI) epi_prefetch(0, epi_res[0], epi_bias[0]);
    wait_vmcnt<0>();  // the clamped re-loads of the loop tail must not land in the epilogue's staging area
  }

  // ---- epilogue through LDS: every lane ends up with 8 consecutive columns of one row, so bias,
  // residual and output move as 16-byte pieces that are contiguous along rows. ----
  // Each wave stages its own WTM x (GA*32) fp32 block (GA column tiles per pass) in LDS that the
  // k-loop no longer needs; rows are padded by 4 floats so the 16-byte transposing writes of 16
  // lanes fall into distinct banks.
  __syncthreads();                 // every wave has finished reading the k-loop buffers
  DS_STAMP(2);
  float* stg = reinterpret_cast<float*>(lds) + wave * (WTM * RSTR);
#pragma unroll
  for (int pass = 0; pass < NPASS; ++pass) {
    const int a0 = pass * GA;
    const int ga = (TN - a0) < GA ? (TN - a0) : GA;  // column tiles in this pass (compile-time after unrolling)
    u32x4* resv = epi_res[pass & 1];
    u32x4* biasv = epi_bias[pass & 1];
    // the next pass's residual / bias pieces travel while this pass is transposed and stored
    if (pass + 1 < NPASS) epi_prefetch(a0 + GA, epi_res[(pass + 1) & 1], epi_bias[(pass + 1) & 1]);
    // 1. accumulators -> LDS (transposing): lane holds rows b*32 + lane%32, columns a*32 + 8g + 4*(lane/32) + 0..3
#pragma unroll
    for (int a = 0; a < GA; ++a) {
      if (a >= ga) break;
#pragma unroll
      for (int b = 0; b < TM; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          floatx4 v;
          v[0] = acc[a0 + a][b][4 * g + 0]; v[1] = acc[a0 + a][b][4 * g + 1];
          v[2] = acc[a0 + a][b][4 * g + 2]; v[3] = acc[a0 + a][b][4 * g + 3];
          *reinterpret_cast<floatx4*>(stg + (b * 32 + (lane & 31)) * RSTR + a * 32 + g * 8 + (lane >> 5) * 4) = v;
        }
    }
    // 2. read back row-contiguous: chunk = 8 columns; cpr chunks per row
    const int cpr = ga * 4;
    const int iters = WTM * cpr / 64;
#pragma unroll
    for (int it = 0; it < MAX_ITERS; ++it) {
      if (it >= iters) break;
      const int idx = it * 64 + lane;
      const int r = idx / cpr, ch = idx - r * cpr;
      const int row = row_base + r, n = col_base + a0 * 32 + ch * 8;
      const floatx4 lo = *reinterpret_cast<const floatx4*>(stg + r * RSTR + ch * 8);
      const floatx4 hi = *reinterpret_cast<const floatx4*>(stg + r * RSTR + ch * 8 + 4);
      if (EPI == kEpiPartial) {  // split-K: raw fp32 sums, row-contiguous
        if (row < p.M && n < p.N) {
          float* dst = p.partial + ((size_t)blockIdx.y * p.M + row) * p.N + n;
          *reinterpret_cast<floatx4*>(dst) = lo;
          *reinterpret_cast<floatx4*>(dst + 4) = hi;
        }
        continue;
      }
      const u32x4 bv = biasv[(64 % cpr != 0) ? it : 0];
      float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      u32x4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float e0 = v[2 * j] + bf16_lo(bv[j]);
        float e1 = v[2 * j + 1] + bf16_hi(bv[j]);
        if (p.relu) {
          e0 = fmaxf(e0, 0.f);
          e1 = fmaxf(e1, 0.f);
        }
        e0 += bf16_lo(resv[it][j]);
        e1 += bf16_hi(resv[it][j]);
        o[j] = pack_bf16(e0, e1);
      }
      if (row < p.M && n < p.N) {
        const int hq = p.n_heads * p.head_dim, hkv = p.n_kv_heads * p.head_dim;
        if (EPI == kEpiKvScatter && n >= hq) {  // this step's new K / V row of sequence `row`: straight into its page
          const int which = n >= hq + hkv;
          const int col = n - hq - which * hkv;
          const int head = col / p.head_dim, d = col - head * p.head_dim;
          const int pos = p.ctx_lens[row];
          const int blk = p.block_tables[(size_t)row * p.max_blocks + pos / 16];
          st16((which ? p.v_cache : p.k_cache) + (((size_t)blk * p.n_kv_heads + head) * 16 + (pos % 16)) * p.head_dim + d, o);
        } else {
          const int seg = (n >= p.seg_cols) + (n >= p.seg_cols + p.seg_cols_kv);
          const int ld = seg == 0 ? p.ld_out : p.seg_cols_kv;
          const int first = seg == 0 ? 0 : p.seg_cols + (seg - 1) * p.seg_cols_kv;
          st16(p.out[seg] + (size_t)row * ld + (n - first), o);
        }
      }
    }
  }
  DS_STAMP(3);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int EPI>
static hipError_t launch_dl_epi(GemmParams p, int splits, hipStream_t stream) {
  p.tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N - p.n_base + BN - 1) / BN;
  constexpr size_t lds_bytes = gemm_lds_bytes(BM, BN, STAGES);
  static_assert((size_t)STAGES * (BM + BN) * kBK * sizeof(uint16_t) <= lds_bytes && lds_bytes <= 160 * 1024, "LDS");
  constexpr auto kern = gemm_dl_kernel<BM, BN, WAVES_M, WAVES_N, STAGES, EPI>;
  (void)KernelAttrReg<kern, (int)lds_bytes>::done;
  hipLaunchKernelGGL(kern, dim3(p.tiles_m * p.tiles_n, splits), dim3(64 * WAVES_M * WAVES_N), lds_bytes, stream, p);
  return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool KV_OK>
static hipError_t launch_dl(const GemmParams& p, int splits, hipStream_t stream) {
  if (splits > 1) return launch_dl_epi<BM, BN, WAVES_M, WAVES_N, STAGES, kEpiPartial>(p, splits, stream);
  if (KV_OK && p.k_cache) return launch_dl_epi<BM, BN, WAVES_M, WAVES_N, STAGES, kEpiKvScatter>(p, 1, stream);
  return launch_dl_epi<BM, BN, WAVES_M, WAVES_N, STAGES, kEpiPlain>(p, 1, stream);
}

// Cost model used to pick a tile shape: (rounds of workgroups on 256 CUs, one workgroup per CU) x
// tile area x a per-area factor of the tile shape.  Under sustained matrix load the chip runs at its
// power limit, so a partly filled last round costs less than a full one (the busy CUs clock higher):
// only 30 % of the idle part of the last round is charged.  Factors are measured ratios of time per
// flop: the 256x256 tile moves 23 % fewer operand bytes per flop than 256x160, the 128x128 tile 50 % more.
static double tile_cost(int M, int N, int BM, int BN, double factor) {
  const long tiles = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const double exact = tiles / 256.0;
  const double full = (double)((tiles + 255) / 256);
  const double rounds = tiles <= 256 ? 1.0 : exact + 0.3 * (full - exact);
  return rounds * BM * BN * factor;
}

DS_SWITCH(g_gemm_variant, 0);     // 0 = cost model, 1..5 force a tile
DS_SWITCH(g_gemm_splits, 0);      // 0 = plan, > 0 force the split count
DS_SWITCH(g_gemm_tail_split, 1);  // 0 = never cut a product at a column
DS_SWITCH(g_gemm_cut_cols, 0);    // > 0: cut at this column ...
DS_SWITCH(g_gemm_tail_kind, 0);   // ... with this tile for the rest (1, 2, 7)

struct GemmPlan {
  int variant;  // 1: 256x160, 2: 128x128, 3: 256x256, 4: 64x128, 5: 128x256 (7: 256x128, behind a cut only)
  int splits;
  int cut_cols = 0;     // > 0: the product is cut at this column; [0, cut_cols) on `variant`, the rest on ...
  int tail_variant = 0; // ... this tile, as a second launch
};

// Tile shape by the cost model above; split count so that a launch with few tiles still occupies the
// chip.  Measured on the decode shapes (M <= 256): >= ~100 workgroups of 128 weight rows stream at
// 5-6 TB/s unsplit; 40 tiles need 4-6 splits; more than ~250 workgroups gain nothing.
// Up to 256 rows the product is bound by streaming the weights, not by the matrix cores, and what a launch
// costs is the bytes its busiest compute unit has to pull through its load path (about 35 GB/s per unit,
// activation re-reads out of L2 included): rounds x (weight + activation bytes of a workgroup's K share
// + its partial tile), plus the reduce pass when K is split.  Used where the rule below would start a second,
// mostly empty round (FFN-in of OPT-13B at 256 rows: 320 tiles of 128x128, 111 us; re-planned 77 us).  For
// single-round launches the measured split counts of the rule below beat this model by 5-25 %, so it is
// not applied to them.
static GemmPlan decode_plan(int M, int N, int K) {
  static const int kBm[5] = {0, 256, 128, 256, 64}, kBn[5] = {0, 160, 128, 256, 128};
  const int kt = K / kBK;
  const int max_s = kt / 8 > 0 ? (kt / 8 < 32 ? kt / 8 : 32) : 1;  // at least 8 k-tiles per split
  GemmPlan best{2, 1};
  double best_cost = 1e30;
  for (int v = 1; v <= 4; ++v) {
    const long tm = (M + kBm[v] - 1) / kBm[v], tn = (N + kBn[v] - 1) / kBn[v];
    const double rows = (double)M / tm;  // activation rows a tile really has
    for (int sp = 1; sp <= max_s; ++sp) {
      const long wgs = tm * tn * sp;
      const double rounds = (double)((wgs + 255) / 256);
      double cost = rounds * ((kBn[v] + rows) * ((double)K / sp) * 2.0 + (sp > 1 ? kBm[v] * kBn[v] * 4.0 : 0.0));
      if (sp > 1) cost += (double)sp * M * N * 4.0 / 256.0 + 175e3;  // reduce pass: its reads, and about 5 us
      if (cost < best_cost) {
        best_cost = cost;
        best = GemmPlan{v, sp};
      }
    }
  }
  return best;
}

// Prefill-sized products (more than 256 rows): tile shape, split count and column cut together, by a time
// model fitted to this chip (OPT-13B shapes, 512-2048 rows, weights not resident in any cache).
//  * A workgroup's k-loop costs us_per_kk microseconds per 1000 elements of K when all 256 compute units are
//    busy, plus t0 for its prologue and epilogue (the output burst of a whole round of tiles is bound by write
//    bandwidth: 9 us for 256x256 tiles, 5 us for 256x160).
//  * Fewer workgroups than compute units: the busy ones clock higher (the chip is power-limited under matrix
//    load), so only 30 % of the idle share is charged.  A partly filled round after full ones is charged
//    80 % of its idle share: its tiles cost what the full rounds' tiles cost.
//  * Splitting K pays where the tiles alone leave most of the chip idle - 512 to 1024 rows against 5120
//    output columns: FFN-out of OPT-13B at 512 rows 186 -> 118 us on four splits of 256x160 tiles, at 1024
//    rows 357 -> 202 us on two.  It costs the fp32 partials' round trip (cheap while they fit the caches) and
//    a reduce launch, and is only considered for launches that stay within one round.
//  * Tile quantisation: 2.5 rounds cost nearly 3.  A product may be cut at a column: the leading columns keep
//    the large tile in whole rounds, the rest runs as a second launch on 256x160 or 128x128 tiles (bias,
//    residual and output pointers follow the cut).  FFN-in of OPT-13B at 2048 rows: 383 us whole, 348 us as
//    two rounds of 256x256 tiles plus one of 256x160.
struct TileModel {
  int variant, bm, bn;
  double us_per_kk, t0;
};
static const TileModel kTileModels[] = {{3, 256, 256, 24.2, 11.6}, {1, 256, 160, 16.5, 7.9},
                                        {5, 128, 256, 15.0, 8.0}, {2, 128, 128, 11.5, 6.0},
                                        // for the columns behind a cut only: FFN-in of OPT-13B at 2048 rows ends
                                        // on 4096 columns = one exact round of 256x128 tiles (355 us for the
                                        // product against 362 us with 208 tiles of 256x160).  (A 256x224 tile,
                                        // which makes QKV two exact rounds of 8192 + 7168 columns, measured 2 %
                                        // slower than 1.875 rounds of 256x256 tiles: not kept.)
                                        {7, 256, 128, 14.5, 7.0}};
// time of `tiles` workgroups of tile t over K (one launch, no split)
static double tiles_us(const TileModel& t, long tiles, double K) {
  const double exact = tiles / 256.0, full = (double)((tiles + 255) / 256);
  if (tiles <= 256) return (0.7 + 0.3 * exact) * t.us_per_kk * K * 1e-3 + t.t0;
  return (exact + 0.8 * (full - exact)) * (t.us_per_kk * K * 1e-3 + t.t0);
}
static GemmPlan prefill_plan(int M, int N, int K) {
  const int kt = K / kBK;
  GemmPlan best{1, 1};
  double best_us = 1e30;
  for (const TileModel& t : kTileModels) {
    if (t.variant > 5) continue;
    const long tm = (M + t.bm - 1) / t.bm, tn = (N + t.bn - 1) / t.bn;
    const long tiles = tm * tn;
    for (int sp = 1; sp <= 8; ++sp) {
      if (sp > 1 && (kt / sp < 8 || tiles * sp > 256)) break;
      double us = tiles_us(t, tiles * sp, (double)K / sp);
      if (sp > 1) {  // larger fp32 epilogue, a reduce launch, partials out and back
        const double mn = (double)M * N;
        us += 4.0 + 2.0 + (8.0 * sp + 2.0) * mn / (sp * mn * 4.0 <= 32e6 ? 12e6 : 5e6);
      }
      if (us < best_us) {
        best_us = us;
        best = GemmPlan{t.variant, sp};
      }
    }
    if (!g_gemm_tail_split || (t.variant != 1 && t.variant != 3) || tiles <= 256) continue;
    // cut after c column tiles (whole rounds of the large tile only), the rest on a smaller tile
    for (long c = tn - 1; c >= 1; --c) {
      if ((tm * c) % 256 != 0 && tm * c > 256) continue;
      const long rest = N - c * t.bn;
      if (rest <= 0) continue;
      for (const TileModel& u : kTileModels) {
        if (u.variant != 1 && u.variant != 2 && u.variant != 7) continue;
        if (u.variant == 1 && t.variant == 1) continue;
        if (u.bn > t.bn) continue;
        const long tiles_u = (long)((M + u.bm - 1) / u.bm) * ((rest + u.bn - 1) / u.bn);
        const double us = tiles_us(t, tm * c, K) + tiles_us(u, tiles_u, K) + 3.0;  // a second launch
        if (us < best_us) {
          best_us = us;
          best = GemmPlan{t.variant, 1, (int)(c * t.bn), u.variant};
        }
      }
    }
  }
  if (g_gemm_cut_cols > 0 && g_gemm_cut_cols < N) best = GemmPlan{3, 1, g_gemm_cut_cols, g_gemm_tail_kind};
  return best;
}

static GemmPlan gemm_plan(int M, int N, int K) {
  GemmPlan pl{1, 1};
  if (M > 256 && g_gemm_variant == 0 && g_gemm_splits == 0) return prefill_plan(M, N, K);
  if (M <= 64) {
    pl.variant = 4;
  } else {
    const double c1 = tile_cost(M, N, 256, 160, 1.0);
    const double c2 = tile_cost(M, N, 128, 128, 1.3);
    const double c3 = tile_cost(M, N, 256, 256, 0.9);
    pl.variant = (c3 < c1 && c3 < c2) ? 3 : (c2 < c1 ? 2 : 1);
  }
  if (g_gemm_variant > 0) pl.variant = g_gemm_variant;
  const int bm = pl.variant == 4 ? 64 : ((pl.variant == 2 || pl.variant == 5) ? 128 : 256);
  const int bn = pl.variant == 1 ? 160 : ((pl.variant == 3 || pl.variant == 5) ? 256 : 128);
  const long tiles = (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
  const int kt = K / kBK;
  if (tiles < 100) {
    int s = (int)((200 + tiles / 2) / tiles);
    const int cap = kt / 8 > 0 ? kt / 8 : 1;  // at least 8 k-tiles per split
    if (s > cap) s = cap;
    if (s > 32) s = 32;
    if (s < 1) s = 1;
    pl.splits = s;
  }
  if (g_gemm_splits > 0) pl.splits = g_gemm_splits < kt ? g_gemm_splits : kt;
  // decode-sized launch that would need a second, mostly empty round: re-plan by bytes per compute unit
  if (M <= 256 && tiles * pl.splits > 256 && g_gemm_variant == 0 && g_gemm_splits == 0) return decode_plan(M, N, K);
  return pl;
}

void gemm_describe(int M, int N, int K, int* tile_rows, int* tile_cols, int* splits, int* cut_cols) {
  static const int kBm[6] = {0, 256, 128, 256, 64, 128}, kBn[6] = {0, 160, 128, 256, 128, 256};
  const GemmPlan pl = gemm_plan(M, N, K);
  *tile_rows = kBm[pl.variant];
  *tile_cols = kBn[pl.variant];
  *splits = pl.splits;
  *cut_cols = pl.cut_cols;
}

int gemm_splits(int M, int N, int K) {
  if (M <= 0 || N <= 0 || K < kBK || K % kBK != 0) return 1;
  return gemm_plan(M, N, K).splits;
}

// Bytes of split-K partials a launch with exactly M rows needs.
size_t gemm_workspace_bytes(int M, int N, int K) {
  if (M <= 0 || N <= 0 || K < kBK || K % kBK != 0) return 0;
  const GemmPlan pl = gemm_plan(M, N, K);
  return pl.splits > 1 ? (size_t)pl.splits * M * N * sizeof(float) : 0;
}

hipError_t launch_gemm(const void* X, const void* W, int M, int N, int K, const Epilogue& ep,
                       hipStream_t stream, void* workspace, const SkinnyFused* fused, bool* fused_done) {
  if (fused_done) *fused_done = false;
  if (M <= 0 || N <= 0) return hipSuccess;
  if (K < kBK || K % kBK != 0 || N % 8 != 0 || ep.seg_cols <= 0 || ep.seg_cols % 8 != 0 || ep.seg_cols_kv < 0 ||
      ep.seg_cols_kv % 8 != 0)
    return hipErrorInvalidValue;
  if (ep.residual && ep.seg_cols != N) return hipErrorInvalidValue;
  if (ep.x_ld != 0 && (ep.x_ld < K || ep.x_ld % 8 != 0)) return hipErrorInvalidValue;
  if (ep.out_ld != 0 && (ep.out_ld < N || ep.out_ld % 8 != 0 || ep.seg_cols != N)) return hipErrorInvalidValue;
  // operand offsets inside the kernel are 32-bit element counts
  if ((unsigned long long)M * (ep.x_ld > 0 ? ep.x_ld : K) >= (1ull << 32) || (unsigned long long)N * K >= (1ull << 32))
    return hipErrorInvalidValue;
  GemmParams p;
  p.X = (const uint16_t*)X;
  p.W = (const uint16_t*)W;
  p.bias = (const uint16_t*)ep.bias;
  p.residual = (const uint16_t*)ep.residual;
  for (int i = 0; i < 3; ++i) p.out[i] = (uint16_t*)ep.out[i];
  p.seg_cols = ep.seg_cols;
  p.seg_cols_kv = ep.seg_cols_kv > 0 ? ep.seg_cols_kv : ep.seg_cols;
  p.ldx = ep.x_ld > 0 ? ep.x_ld : K;
  p.ld_out = ep.out_ld > 0 ? ep.out_ld : ep.seg_cols;
  p.ld_res = N;
  p.n_base = 0;
  p.M = M; p.N = N; p.K = K;
  p.relu = ep.relu;
  p.tiles_m = p.tiles_n = 0;
  p.partial = nullptr;
  p.ctx_lens = nullptr; p.block_tables = nullptr; p.max_blocks = 0;
  p.k_cache = nullptr; p.v_cache = nullptr; p.n_heads = 0; p.n_kv_heads = 0; p.head_dim = 0;
#ifdef DS_DEV_SWITCHES
  p.dbg = g_gemm_dbg;
#endif
  GemmPlan pl = gemm_plan(M, N, K);
  if (pl.splits > 1 && workspace == nullptr) pl.splits = 1;  // no room for partials: slower, still right
  if (pl.splits > 1 && ep.out_ld != 0) return hipErrorInvalidValue;  // the reduce pass writes dense rows
  const bool want_kv = fused && fused->kind == SkinnyFused::kKvAppend && ep.seg_cols == N && !ep.relu &&
                       !ep.residual && N == (fused->n_heads + 2 * fused->n_kv_heads) * fused->head_dim &&
                       fused->head_dim % 8 == 0;
  if (pl.splits > 1) {
    p.partial = (float*)workspace;
  } else if (want_kv && (pl.variant == 2 || pl.variant == 4)) {
    // unsplit (decode-sized tiles only): the tile kernel's own epilogue scatters K and V into the cache
    p.ctx_lens = fused->ctx_lens; p.block_tables = fused->block_tables; p.max_blocks = fused->max_blocks;
    p.k_cache = (uint16_t*)fused->k_cache; p.v_cache = (uint16_t*)fused->v_cache;
    p.n_heads = fused->n_heads; p.n_kv_heads = fused->n_kv_heads; p.head_dim = fused->head_dim;
    if (fused_done) *fused_done = true;
  }
  hipError_t e;
  if (pl.cut_cols > 0 && pl.splits == 1 && !p.k_cache) {
    // Leading columns on the large tile in whole rounds of 256 workgroups, the rest on a smaller tile: two
    // launches over disjoint column ranges [0, cut) and [cut, N) of the same product (same operands, bias,
    // residual and output segments; only the column range differs).
    GemmParams a = p, b = p;
    a.N = pl.cut_cols;
    b.n_base = pl.cut_cols;
    e = pl.variant == 3 ? launch_dl<256, 256, 2, 2, 2, false>(a, 1, stream)
                        : launch_dl<256, 160, 4, 1, 3, false>(a, 1, stream);
    if (e != hipSuccess) return e;
    switch (pl.tail_variant) {
      case 1: return launch_dl<256, 160, 4, 1, 3, false>(b, 1, stream);
      case 7: return launch_dl_epi<256, 128, 4, 1, 3, kEpiPlain>(b, 1, stream);
      default: return launch_dl<128, 128, 2, 2, 3, true>(b, 1, stream);
    }
  }
  switch (pl.variant) {
    case 5: e = launch_dl<128, 256, 2, 2, 3, false>(p, pl.splits, stream); break;
    case 4: e = launch_dl<64, 128, 1, 4, 3, true>(p, pl.splits, stream); break;
    case 3: e = launch_dl<256, 256, 2, 2, 2, false>(p, pl.splits, stream); break;
    case 2: e = launch_dl<128, 128, 2, 2, 3, true>(p, pl.splits, stream); break;
    default: e = launch_dl<256, 160, 4, 1, 3, false>(p, pl.splits, stream); break;
  }
  if (e != hipSuccess) return e;
  if (pl.splits > 1) e = launch_splitk_reduce(p.partial, pl.splits, M, N, ep, fused, fused_done, stream);
  return e;
}

}  // namespace ds
