// Causal attention inside each packed request, flash style on the matrix cores.
//
// A workgroup (4 waves) owns 128 consecutive queries of one (request, head);
// wave w owns 32 of them.  Keys/values are visited in tiles of 64.  The score
// tile is computed transposed, S^T[key, query] = K Q^T, so that in the MFMA
// result layout every lane holds scores of ONE query (lane % 32): the running
// max / sum / rescale factors are per-lane scalars, and the probabilities are
// already in the register layout the second product O^T[d, query] = V^T P^T
// needs as its column operand - no shuffles, no LDS round trip for P.
// K and V tiles arrive row-major by direct global->LDS loads into two buffers (tile i+1 lands while tile i
// is multiplied); the V^T fragments of the second product come out of the row-major V tile through the
// transposing LDS read.
#include "common.h"
#include "kernels.h"

namespace ds {

constexpr int kAttThreads = 256;
constexpr int kAttQ = 128;    // queries per workgroup
constexpr int kAttKV = 64;    // keys per tile
constexpr float kSlack = 8.f;   // exponent headroom before the softmax reference point is moved

#ifdef DS_DEV_SWITCHES
// timing harness builds only: 16 wall-clock stamps (100 MHz) per workgroup - entry, first tile landed, the end
// of each of the first 12 tiles, exit - and the tile count
unsigned long long* g_attn_dbg = nullptr;
#define DS_ATT_DBG_PARAM , unsigned long long* dbg
#define DS_ATT_DBG_ARG , g_attn_dbg
#define DS_ATT_STAMP(i)                                                                          \
  do {                                                                                           \
    if (dbg && threadIdx.x == 0) dbg[(size_t)blockIdx.x * 16 + (i)] = __builtin_amdgcn_s_memrealtime(); \
  } while (0)
#else
#define DS_ATT_DBG_PARAM
#define DS_ATT_DBG_ARG
#define DS_ATT_STAMP(i)
#endif

template <int HD>
__global__ __launch_bounds__(kAttThreads) __attribute__((amdgpu_waves_per_eu(2))) void prefill_attention_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ cu_seqlens, uint16_t* __restrict__ o, int n_heads, int kv_group,
    float scale_log2e,
    int n_pairs, int pairs_per_xcd, int n_qt, int fold DS_ATT_DBG_PARAM) {
  constexpr int DSTEPS = HD / 16;   // MFMA k-steps over the head dimension
  constexpr int DT = HD / 32;       // 32-row tiles of O^T
  constexpr int CPR = HD / 8;       // 16-byte chunks per K/V row
  // Two LDS buffers of [K tile | V tile], each tile 64 rows of HD elements, row-major and unpadded: the tiles
  // arrive by direct global->LDS loads (a wave-level load drops 64 consecutive 16-byte pieces), so bank conflicts
  // are avoided by storing chunk c of row r at position c ^ swizzle(r), applied on the global side of the load.
  //   K (16-byte fragment reads of 32 consecutive rows at one chunk index): rows of 256 bytes r & 15, of 128 bytes (r >> 1) & 7.
  //   V (transposing 8-byte reads: 4 consecutive rows x 4 consecutive chunks per half wave): (r & 3) << 2 for
  //   256-byte rows; ((r >> 1) & 1) << 2 for 128-byte rows, whose neighbours already sit in different bank halves.
  constexpr int TILE_ELEMS = kAttKV * HD, BUF_ELEMS = 2 * TILE_ELEMS;
  extern __shared__ __attribute__((aligned(1024))) uint16_t att_lds[];

  // Workgroups reach the chip's eight partitions (each with its own L2) round-robin in launch
  // order, so id % 8 names the partition and id / 8 the order inside it.  A (request, head) pair is
  // pinned to one partition.
  //  * While the K/V that the resident workgroups re-read between them stays in the last-level cache: one tile per
  //    workgroup, ordered heaviest first across all pairs (longest-first balances the tail, and workgroups that
  //    follow each other have equal work).
  //  * Beyond that: the workgroups of one pair run back to back, so its K/V stay in that partition's L2 while they are
  //    re-read, and each takes TWO query tiles, tile nq-1-r and then its mirror image r, so that all workgroups
  //    of a sequence have the same nq+1 key tiles of work.  Equal work matters more than it seems: inside a
  //    partition workgroups are dealt to the shader engines in launch order, a full engine holds up the ones
  //    behind it, and with one tile per workgroup (2 .. 2 nq key tiles, in a fixed pattern) a compute unit had
  //    fewer than two workgroups resident for 40 % of the launch while thousands were still queued.
  const int id = blockIdx.x;
  const int xcd = id & 7, slot = id >> 3;
  const int n_ranks = fold ? (n_qt + 1) / 2 : n_qt;   // workgroups per pair
  const int pl = fold ? slot / n_ranks : slot % pairs_per_xcd;
  const int rank = fold ? slot % n_ranks : slot / pairs_per_xcd;
  const int pair = pl * 8 + xcd;
  if (pair >= n_pairs) return;
  const int seq = pair / n_heads;
  const int head = pair - seq * n_heads;
  const int start = cu_seqlens[seq];
  const int len = cu_seqlens[seq + 1] - start;
  int qt, qt_next = -1;
  if (fold) {
    const int nq = (len + kAttQ - 1) / kAttQ;   // this sequence's query tiles
    if (rank >= (nq + 1) / 2) return;
    qt = nq - 1 - rank;                         // the heavy one first
    if (qt != rank) qt_next = rank;
  } else {
    qt = n_qt - 1 - rank;                       // heaviest query tile (most keys) first
    if (qt * kAttQ >= len) return;
  }
  DS_ATT_STAMP(0);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hl = lane >> 5, lq = lane & 31;
  const size_t h = (size_t)n_heads * HD;                // q, o row length
  const size_t hk = (size_t)(n_heads / kv_group) * HD;  // k, v row length: kv_group query heads share a key/value head
  const uint16_t* kbase = k + (size_t)start * hk + (size_t)(head / kv_group) * HD;
  const uint16_t* vbase = v + (size_t)start * hk + (size_t)(head / kv_group) * HD;

  // Tile i+1 is requested (global -> LDS, no registers) into the other buffer before tile i is multiplied; one
  // workgroup barrier per tile: it closes the reads of tile i and publishes tile i+1.
  constexpr int NLD = kAttKV * CPR / kAttThreads;   // wave-level loads per wave, tile and operand (4 or 2)
  constexpr int RPL = 64 / CPR;                     // tile rows per wave-level load (4 or 8)
  // Wave-level load j of a wave drops 64 consecutive 16-byte pieces: tile rows ld_row0 + j RPL .. + RPL - 1 with
  // all their chunks; the lane's piece is chunk ld_c of its row and comes from source chunk ld_c ^ swizzle(row).
  // With the row numbers written out the K swizzle is (low bits of the lane's row) ^ 4j, the V swizzle the same for
  // all j.  A tile that lies inside the request is fetched from one scalar base plus 32-bit lane offsets that do not
  // change from tile to tile; only the last tile needs its rows clamped.
  const int ld_sub = lane / CPR, ld_c = lane % CPR;
  const int ld_row0 = wave * NLD * RPL + ld_sub;
  const int ld_kcol0 = (ld_c ^ (CPR == 16 ? ld_sub : (ld_sub >> 1))) * 8;
  const int ld_vcol = (ld_c ^ (CPR == 16 ? (ld_sub << 2) : (((ld_sub >> 1) & 1) << 2))) * 8;
  uint32_t ld_koff[NLD], ld_voff[NLD];   // element offsets from the tile's first row
#pragma unroll
  for (int j = 0; j < NLD; ++j) {
    ld_koff[j] = (uint32_t)(ld_row0 + j * RPL) * (uint32_t)hk + (uint32_t)(ld_kcol0 ^ (32 * j));
    ld_voff[j] = (uint32_t)(ld_row0 + j * RPL) * (uint32_t)hk + (uint32_t)ld_vcol;
  }
  auto request = [&](int kv0, int buf) {
    uint16_t* kdst = att_lds + buf * BUF_ELEMS + (wave * NLD) * 512;
    if (kv0 + kAttKV <= len) {
      const uint16_t* kt = kbase + (size_t)kv0 * hk;
      const uint16_t* vt = vbase + (size_t)kv0 * hk;
#pragma unroll
      for (int j = 0; j < NLD; ++j) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kt + ld_koff[j]),
                                         (__attribute__((address_space(3))) void*)(kdst + j * 512), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vt + ld_voff[j]),
                                         (__attribute__((address_space(3))) void*)(kdst + TILE_ELEMS + j * 512), 16, 0, 0);
      }
    } else {   // rows past the end repeat the last key (they are masked out below)
#pragma unroll
      for (int j = 0; j < NLD; ++j) {
        const size_t row = (size_t)min(kv0 + ld_row0 + j * RPL, len - 1) * hk;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kbase + row + (ld_kcol0 ^ (32 * j))),
                                         (__attribute__((address_space(3))) void*)(kdst + j * 512), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vbase + row + ld_vcol),
                                         (__attribute__((address_space(3))) void*)(kdst + TILE_ELEMS + j * 512), 16, 0, 0);
      }
    }
  };
  auto wait_loads = [] {  // s_waitcnt vmcnt(0) only: vmcnt[3:0] | expcnt=7 | lgkmcnt=15 | vmcnt[5:4] in bits 15:14
    __builtin_amdgcn_s_waitcnt((0x7 << 4) | (0xf << 8));
  };
#ifdef DS_DEV_SWITCHES
  int dbg_tiles = 0;
#endif
  for (;;) {   // one query tile, or two
    const int q0 = qt * kAttQ;
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
#ifdef DS_DEV_SWITCHES
    dbg_tiles += n_tiles;
#endif

    request(0, 0);
    wait_loads();
    __syncthreads();
    DS_ATT_STAMP(1);

    const int kswz = CPR == 16 ? (lq & 15) : ((lq >> 1) & 7);   // K fragment rows are u*32 + lq
    for (int tile = 0; tile < n_tiles; ++tile) {
      const int kv0 = tile * kAttKV;
      const uint16_t* ks = att_lds + (tile & 1) * BUF_ELEMS;
      const uint16_t* vs = ks + TILE_ELEMS;
      // the other buffer was last read in iteration tile-1, which every wave left through the barrier below
      if (tile + 1 < n_tiles) request(kv0 + kAttKV, (tile + 1) & 1);
      // nothing to multiply if every key of this tile is in the future of this wave's queries, or the wave has no
      // query at all; the wave still takes part in the loads and the barrier
      if (kv0 > qw0 + 31 || qw0 >= len) {
        wait_loads();
        __syncthreads();
        if (tile < 12) DS_ATT_STAMP(2 + tile);
        continue;
      }

      // ---- S^T = K Q^T : two 32-key row tiles ----
      // The two row tiles advance together, so that consecutive matrix instructions write different
      // accumulators (a chain on one accumulator waits out the full latency of every instruction), and the K
      // fragments are requested from LDS half a tile ahead of their use (scheduling fences keep the compiler
      // from sinking each read down to its instruction, which exposes the LDS latency sixteen times).
      floatx16 sacc[2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[u][r] = 0.f;
      {
        constexpr int HS = DSTEPS / 2;
        const uint16_t* kr0 = ks + lq * HD;   // chunk 2 st + hl of rows lq and 32 + lq (same swizzle key)
        const uint16_t* kr1 = kr0 + 32 * HD;
        auto kcol = [&](int st) { return ((2 * st + hl) ^ kswz) * 8; };
        bf16x8 kf[2][HS];
#pragma unroll
        for (int st = 0; st < HS; ++st) {
          kf[0][st] = *reinterpret_cast<const bf16x8*>(kr0 + kcol(st));
          kf[1][st] = *reinterpret_cast<const bf16x8*>(kr1 + kcol(st));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < HS; ++st) {
          sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][st], qf[st], sacc[0], 0, 0, 0);
          sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][st], qf[st], sacc[1], 0, 0, 0);
          kf[0][st] = *reinterpret_cast<const bf16x8*>(kr0 + kcol(st + HS));
          kf[1][st] = *reinterpret_cast<const bf16x8*>(kr1 + kcol(st + HS));
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int st = 0; st < HS; ++st) {
          sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][st], qf[st + HS], sacc[0], 0, 0, 0);
          sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][st], qf[st + HS], sacc[1], 0, 0, 0);
        }
      }
      // ---- causal mask + running softmax; element r of tile u is key kv0 + 32u + 8(r/4) + 4hl + r%4 ----
      // Only a tile that reaches past the wave's first query needs the mask (wave-uniform choice).
      if (kv0 + kAttKV - 1 > qw0) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kv0 + u * 32 + (r >> 2) * 8 + hl * 4 + (r & 3);
            if (key > my_q) sacc[u][r] = -INFINITY;
          }
      }
      float tmax = -INFINITY;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, sacc[u][r]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      // The reference point m_run of the exponentials only has to keep them in range, so it is moved
      // (and the accumulators rescaled) only when some query's maximum grew by more than kSlack in
      // the exponent: probabilities then stay below 2^kSlack and the final quotient is unchanged.
      if (__builtin_amdgcn_ballot_w64(tmax * scale_log2e > m_run * scale_log2e + kSlack) != 0) {
        const float m_new = fmaxf(m_run, tmax);  // finite: key kv0 is visible to every query of the wave
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
        l_run *= alpha;
        m_run = m_new;
#pragma unroll
        for (int d = 0; d < DT; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[d][r] *= alpha;
      }
      const float mb = m_run * scale_log2e;
      // Two probabilities at a time: exponentials, one bf16 pair, and the pair's sum added to the running sum by a
      // dot product with (1, 1) - the sum then counts exactly the rounded values the second product multiplies.
      float psum = 0.f;
      u32x4 pw[4];  // pw[2u+v]: column operand of PV step (u,v), as bf16 pairs
      bf16x2 ones;
      ones[0] = (__bf16)1.f;
      ones[1] = (__bf16)1.f;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float pa = __builtin_amdgcn_exp2f(sacc[u][r] * scale_log2e - mb);
          const float pb = __builtin_amdgcn_exp2f(sacc[u][r + 1] * scale_log2e - mb);
          bf16x2 pr;
          pr[0] = (__bf16)pa;
          pr[1] = (__bf16)pb;
          psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
          pw[2 * u + (r >> 3)][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, pr);
        }
      l_run += psum;

      // ---- O^T += V^T P^T.  PV step (u,v) contracts keys 32u+16v + {0..3, 8..11} + 4hl ----
      // The V^T fragments come out of the row-major tile through the transposing LDS read: in a group of 16
      // lanes, lane j hands in the address of 4 consecutive d of key j / 4 (16 d in all, 4 keys), and lane i
      // gets back the 4 keys at d = i.  Groups 0, 1 serve d 0..15, 16..31 of key group hl = 0, groups 2, 3 of hl = 1.
      const int i16 = lane & 15;
      const int vswz = CPR == 16 ? ((i16 >> 2) << 2) : (((i16 >> 3) & 1) << 2);   // rows are 4 hl + i16/4 + multiples of 8
      const uint16_t* vfrag = vs + (4 * hl + (i16 >> 2)) * HD + (i16 & 1) * 4;
      const int vchunk = 2 * ((lane >> 4) & 1) + ((i16 & 3) >> 1);                 // + 4 d: 16-byte chunk of this lane's 4 d
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int vv = 0; vv < 2; ++vv) {
          const uint16_t* vstep = vfrag + (u * 32 + vv * 16) * HD;
#pragma unroll
          for (int d = 0; d < DT; ++d) {
            typedef short short4v __attribute__((ext_vector_type(4)));
            typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;
            const int col = ((4 * d + vchunk) ^ vswz) * 8;
            const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vstep + col));
            const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vstep + 8 * HD + col));
            u32x4 packed;
            const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
            packed[0] = l2[0]; packed[1] = l2[1]; packed[2] = h2[0]; packed[3] = h2[1];
            oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, packed), __builtin_bit_cast(bf16x8, pw[2 * u + vv]), oacc[d], 0, 0, 0);
          }
        }
      wait_loads();     // this wave's share of tile i+1 has landed
      __syncthreads();  // ... and everybody's; and every wave is done reading tile i
      if (tile < 12) DS_ATT_STAMP(2 + tile);
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
    if (qt_next < 0) break;
    qt = qt_next;   // the last tile's barrier closed all reads of both buffers: the next tile may fill them
    qt_next = -1;
  }
  DS_ATT_STAMP(14);
#ifdef DS_DEV_SWITCHES
  if (dbg && threadIdx.x == 0) dbg[(size_t)blockIdx.x * 16 + 15] = (unsigned long long)dbg_tiles;
#endif
}

DS_SWITCH(g_attn_force_order, -1);  // 0/1 force one / two query tiles per workgroup, -1 choose by grid size

hipError_t launch_prefill_attention(const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                                    int B, int t, int max_seqlen, int n_heads, int n_kv_heads, int head_dim, void* o,
                                    hipStream_t stream) {
  if (B <= 0 || max_seqlen <= 0) return hipSuccess;
  if (n_kv_heads <= 0 || n_heads % n_kv_heads != 0) return hipErrorInvalidValue;
  const int kv_group = n_heads / n_kv_heads;
  const int n_qt = (max_seqlen + kAttQ - 1) / kAttQ;
  const long n_pairs = (long)B * n_heads;
  const long pairs_per_xcd = (n_pairs + 7) / 8;
  // One query tile per workgroup, heaviest first over all pairs, while the K/V that the resident workgroups
  // (two per compute unit, 256 units) re-read between them fits the last-level cache with room to spare: workgroups
  // that follow each other then have equal work, which keeps every shader engine supplied.  Beyond that (measured
  // between 150 and 170 MB) the re-reads go to HBM and the launch becomes bandwidth-bound: then a pair's
  // workgroups run back to back on their partition and take two tiles each.
  //   2 x 2048 tokens, 40 heads (84 MB): 105 us one tile per workgroup, 123 us two; 8 x 2048 (335 MB): 589 / 458 us.
  const long wgs_single = 8 * pairs_per_xcd * n_qt;
  const double kv_bytes = 4.0 * t * n_kv_heads * head_dim * (n_pairs > 512 ? 512.0 / n_pairs : 1.0);
  const int fold = g_attn_force_order >= 0 ? g_attn_force_order : (wgs_single > 2 * 512 && kv_bytes > 160e6 ? 1 : 0);
  const long wgs = fold ? 8 * pairs_per_xcd * ((n_qt + 1) / 2) : wgs_single;
  if (wgs > 0x7fffffffL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)wgs);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
  // two buffers of [64 K rows | 64 V rows] of head_dim bf16
  const size_t lds_bytes = (size_t)2 * 2 * kAttKV * head_dim * sizeof(uint16_t);
  if (head_dim == 128) {
    (void)KernelAttrReg<prefill_attention_kernel<128>, 2 * 2 * kAttKV * 128 * (int)sizeof(uint16_t)>::done;
    hipLaunchKernelGGL(prefill_attention_kernel<128>, grid, dim3(kAttThreads), lds_bytes, stream, (const uint16_t*)q,
                       (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, (uint16_t*)o, n_heads, kv_group, scale_log2e,
                       (int)n_pairs, (int)pairs_per_xcd, n_qt, fold DS_ATT_DBG_ARG);
  } else if (head_dim == 64) {
    hipLaunchKernelGGL(prefill_attention_kernel<64>, grid, dim3(kAttThreads), lds_bytes, stream, (const uint16_t*)q,
                       (const uint16_t*)k, (const uint16_t*)v, cu_seqlens, (uint16_t*)o, n_heads, kv_group, scale_log2e,
                       (int)n_pairs, (int)pairs_per_xcd, n_qt, fold DS_ATT_DBG_ARG);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ds
