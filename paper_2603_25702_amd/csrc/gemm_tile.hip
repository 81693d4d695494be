// LDS-tiled MFMA GEMM on the packed bf16 weights for windows of more than 32 rows:
//   Y[m, n] = sum_k X[m, k] W[n, k]
// (verifier / draft forwards of the batched configurations, the prompt prefill, and the grouped
// expert GEMMs of the MoE FFN).
//
// A workgroup of eight wavefronts (one workgroup per compute unit) owns a tile of 128 rows x 256 output features
// and walks K in steps of 64.  The wavefronts stand side by side: each computes all 128 rows x 32 features (8 x 2
// MFMA tiles; for the gate/up pair of SwiGLU 16 features of each matrix, so a workgroup tile is 128 x 128 there).
// Every weight operand is then requested by exactly one wavefront, straight from the packed copy, where one
// wavefront-wide 16-byte load is a complete A operand of v_mfma_f32_16x16x32_bf16, through a ring of three
// register stages: while a step multiplies out of one stage, the stage of the step before is refilled for the
// step after the next (HBM latency is more than a step of MFMA work).  (With the wavefronts 2 x 4 on 64 x 64
// each, every weight operand was requested twice per compute unit: 80 KB per step through an address path of
// 64 bytes per clock.)  The activation tile is loaded once per compute unit and goes through LDS (three buffers,
// rows padded to 144 bytes per plane so that the 16-byte operand reads of a wavefront hit 64 distinct banks);
// all eight wavefronts read all of it, four operand reads ahead of the MFMA pair that uses them.  All memory
// requests of a step are issued one at a time between its MFMA pairs.  (A four-wavefront variant on 128 x 128
// tiles, two workgroups per compute unit, is kept as a tuning aid.)
//
// K can be split over blockIdx.z when the tiles alone would leave compute units idle (few rows, narrow
// outputs): every split writes its accumulators as an fp32 partial in register order (write-through
// stores) and counts itself in at the tile's counter.  The merge is shared: split z finishes every KS-th
// accumulator of the tile (adds the KS partials in split order, runs the epilogue), after a short bounded
// wait for the other splits; all of a split's partials of all splits are requested at once, so the merge
// is one memory round trip per workgroup, and KS compute units share it.  Nothing depends on that wait
// succeeding: a split that gives up says so in the counter word and leaves, and the split that arrives
// last finishes its own share and every share given up before its arrival (a split that gives up after
// the last arrival finds everybody there and finishes its own share after all).  Launches with more
// workgroups than compute units do not wait at all (the last arrival finishes the whole tile).  Every sum
// is formed in split order, so the result does not depend on who forms it.
//
// blockIdx.y covers the row tiles the host expects (m_hint); a workgroup walks on to the row tiles beyond
// that if the device-side row count is larger.  The usual launch therefore has no workgroup without rows:
// the hardware deals workgroups to the shader engines in turn whether they exit at once or not, and
// launches with such workgroups in between were measured to leave a fifth of the compute units empty
// while others held two workgroups one after the other.
//
// The prologue / epilogues are the ones of the streaming kernel (same argument block): 1/rms from
// the producer's partial sums of squares, fp32 store, residual add with the operand and partial
// sums of the next norm, SwiGLU, RoPE + q/k/v split.  In grouped mode a row tile belongs to one
// expert: rows are gathered through the expert-sorted slot list and the down projection scatters
// its result, scaled by the routing weight, to the (token, slot) row it came from.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

#include <algorithm>
#include <type_traits>
#include <stdlib.h>

namespace s2d2 {

static constexpr int TM = 128, TK = 64;
// Tuning constants of the K loop (measured on the batched configurations: 3 to 6 weight stages and 2 to 8 operand
// reads in flight gave the same times within the run-to-run spread)
#ifndef S2D2_TILE_WS
#define S2D2_TILE_WS 3   // weight stages in flight
#endif
#ifndef S2D2_TILE_PD
#define S2D2_TILE_PD 4   // LDS operand reads in flight per wavefront
#endif
#ifdef S2D2_KERNEL_TIMING
__device__ unsigned long long g_tile_ts[1024];   // [128 + 3 id + k]: start, loop end, share known of every workgroup of the last down projection
// stamps of the workgroup of column tile 0, row tile 0, split 0 in [slot * 24 + k], of the last column tile's last split
// in [slot * 24 + 8 + k]; slot = epilogue kind, 4 = residual add with K <= 4096 (output projection)
#define S2D2_TTS(k) do { if (threadIdx.x == 0 && ty == 0) { \
    const int slot_ = (EPI == SEPI_ADD_F32 && a.K <= 4096) ? 4 : EPI; \
    if (bx == 0 && z == 0) g_tile_ts[slot_ * 24 + (k)] = wall_clock64(); \
    if (bx == ncol - 1 && z == KS - 1) g_tile_ts[slot_ * 24 + 8 + (k)] = wall_clock64(); } \
  if (threadIdx.x == 0 && EPI == SEPI_ADD_F32 && a.K > 4096 && ((k) == 0 || (k) == 2 || (k) == 3)) { \
    const int id_ = bx + ncol * (ty + (int)gridDim.y * z); if (id_ < 256) g_tile_ts[128 + 3 * id_ + ((k) == 0 ? 0 : (k) - 1)] = wall_clock64(); } } while (0)
// shader-clock sums over the K steps of the gate / up workgroup of tile (0, 0), per wavefront, in [896 + 16 wave + k]:
// 8: whole steps, 15: number of steps; with S2D2_STEP_EIGHTHS=1 also k < 8: eighth k of the step's MFMA pairs (then
// 8 holds the rest; every stamp waits for the LDS reads in flight, so the eighths cost about 35 clocks each)
#ifndef S2D2_STEP_EIGHTHS
#define S2D2_STEP_EIGHTHS 0
#endif
#define S2D2_STEP_CLK(k) do { __builtin_amdgcn_sched_barrier(0); const unsigned long long c_ = clock64(); \
    if (k) step_sum[(k) - 1] += c_ - step_c; else { step_sum[15] += 1; if (step_c) step_sum[8] += c_ - step_c; } step_c = c_; __builtin_amdgcn_sched_barrier(0); } while (0)
#else
#define S2D2_TTS(k) do {} while (0)
#define S2D2_STEP_CLK(k) do {} while (0)
#define S2D2_STEP_EIGHTHS 0
#endif

// SPLIT: the activations come as a high- and a low-order bf16 plane (16 significant bits); both planes
// of a row sit side by side in LDS and every weight operand is multiplied with both.
// One row tile (index ty) of the workgroup's column tile and K split; false: there is no such row tile.
template <int EPI, int PRO, int OPM, int WC>
// z of KS: this workgroup's share of K; ncol: column tiles of the launch (numbering of the tiles' counters and
// partials); wait_ok: every workgroup of the launch is resident at once, so the splits of a tile may wait for each other;
// same_rows: the row maps in LDS are already those of row tile ty (the workgroup's previous item had the same rows).
__device__ __forceinline__ bool gemm_tile_body(const GemmStreamArgs& a, const int bx, const int ty, const int z, const int KS,
                                               const int ncol, const bool wait_ok, const bool same_rows) {
  constexpr bool SPLIT = OPM == OPM_BF16X2;       // the activations come as two bf16 planes
  constexpr int NTH = 128 * WC;                   // 2 WC wavefronts side by side, each all 128 rows x 32 features
  constexpr int RBN = TM / 16, TN = 2;            // 16-row blocks and 16-feature accumulator columns of a wavefront
  constexpr int XI = 1024 / NTH;                  // 16-byte chunks of an activation plane tile per thread
  constexpr int XD = 2;                           // register sets of the activation tile on its way to LDS
  constexpr int NACC = EPI == SEPI_SWIGLU ? 2 : 1;
  constexpr int FT = TN / NACC;                   // feature tiles per wavefront and matrix; FT * NACC = TN accumulator columns
  constexpr int WS = S2D2_TILE_WS;                // weight stages in flight
  constexpr int XROW = (SPLIT ? 256 : 128) + 16;  // bytes per LDS row: 64 bf16 per plane + 16 bytes of padding
  constexpr int XBUF = TM * XROW;                 // bytes of one activation tile in LDS
  extern __shared__ __align__(16) uint8_t s_xd[];   // three activation tiles (dynamic: 102 KB with two planes)
  __shared__ int s_xrow[TM], s_orow[TM];
  __shared__ float s_rs[TM];
  __shared__ int s_share;

  // (the thread index passes through an opaque statement: otherwise everything that depends on the lane alone is
  // computed ahead of the loop over row tiles, for all epilogues at once, and spilled across the K loop)
  int tid_ = threadIdx.x;
  asm volatile("" : "+v"(tid_));
  const int tid = tid_, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, f = lane & 15;
  int m0, Mloc, expert = 0;
  if (a.grouped != GROUP_NONE) {
    if (ty >= *a.n_tiles) return false;
    expert = a.tile_expert[ty];
    m0 = a.tile_row0[ty];
    Mloc = a.tile_rows[ty];
  } else {
    const int M = *a.m_count;
    m0 = ty * TM;
    if (m0 >= M) return false;
    Mloc = min(TM, M - m0);
  }
  S2D2_TTS(0);
  const int KT = a.KT;
  // live 16-row blocks of this wavefront's 64 rows, as a scalar: the skips in the K loop are then plain scalar
  // branches and not execution-mask regions
  const int rb_live = __builtin_amdgcn_readfirstlane(min(RBN, (Mloc + 15) >> 4));
  const int nt0 = (bx * (2 * WC) + wave) * FT;

  // ---- the weights of the first steps: their addresses need no row map, and their way from memory is the longest
  // of the prologue; they are requested below while the row maps' partial sums are on their way ----
  const int nk = (a.K + TK - 1) / TK;
  const int kb0 = (int)((long long)z * nk / KS), kb1 = (int)((long long)(z + 1) * nk / KS);   // this split's K steps
  const u32x4_t* wp[TN];
#pragma unroll
  for (int t = 0; t < FT; ++t) {
    const int nt = min(nt0 + t, a.NT - 1);
    wp[t * NACC] = (const u32x4_t*)a.Wp + (size_t)expert * a.expert_stride + (size_t)nt * KT * 64 + lane;
    if (NACC == 2) wp[t * NACC + 1] = (const u32x4_t*)a.Wp2 + (size_t)expert * a.expert_stride + (size_t)nt * KT * 64 + lane;
  }
  u32x4_t wst[WS][2][TN];
  auto load_w1 = [&](u32x4_t& w, int kb, int k2, int t) __attribute__((always_inline)) {
    const int kt = min(kb * 2 + k2, KT - 1);   // past the end: some valid tile, multiplied with zeros
    w = wp[t][(size_t)kt * 64];   // (no non-temporal hint here: the other row tiles re-read the weights through L2; with it the GEMMs of the batched configurations took 8-11 % longer)
  };

  // ---- row maps: source row of X, row of the partial sums of squares, destination row, scale ----
  {
    constexpr int TPR = NTH / TM;           // threads per row
    const int r = tid / TPR, hf = tid % TPR;
    int xrow = -1, orow = -1, ssrow = 0;
    float ow = 1.f;
    if (r < Mloc && !same_rows) {
      const int s = m0 + r;
      if (a.grouped == GROUP_GATHER) {          // expert gate/up: X row of the token, output in sorted order
        xrow = a.sorted[s] / a.top_k; ssrow = xrow; orow = s;
      } else if (a.grouped == GROUP_SCATTER) {  // expert down: X in sorted order, output to the (token, slot) row
        xrow = s; orow = a.sorted[s]; ow = a.route_w[orow];
      } else {
        xrow = a.gather ? a.gather[s] : s; ssrow = xrow; orow = s;
      }
    }
    // 1/rms from the producer's partial sums of squares: independent 16-byte loads, 16 in flight per thread and round
    // (one round up to 64 TPR partials per row), not a chain of L2 round trips
    const float* pp = PRO == SPRO_BF16S ? a.ss_part + (size_t)ssrow * a.ss_stride : nullptr;
    const bool vec = PRO == SPRO_BF16S && (a.ss_count & 3) == 0 && (a.ss_stride & 3) == 0;
    const int n4 = (PRO == SPRO_BF16S && r < Mloc && vec && !same_rows) ? a.ss_count >> 2 : 0;
    float4 t[16];
    if (PRO == SPRO_BF16S) {
#pragma unroll
      for (int j = 0; j < 16; ++j) t[j] = (hf + TPR * j < n4) ? ((const float4*)pp)[hf + TPR * j] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int st_ = 0; st_ < WS - 1; ++st_)
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
        for (int tt = 0; tt < TN; ++tt) load_w1(wst[st_][k2][tt], kb0 + st_, k2, tt);
    float rs = ow;
    if (PRO == SPRO_BF16S) {
      float v = 0.f;
#pragma unroll
      for (int j = 0; j < 16; ++j) v += (t[j].x + t[j].y) + (t[j].z + t[j].w);
      for (int i0 = hf + 16 * TPR; i0 < n4; i0 += 16 * TPR) {
#pragma unroll
        for (int j = 0; j < 16; ++j) t[j] = (i0 + TPR * j < n4) ? ((const float4*)pp)[i0 + TPR * j] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int j = 0; j < 16; ++j) v += (t[j].x + t[j].y) + (t[j].z + t[j].w);
      }
      if (!vec && r < Mloc && !same_rows)
        for (int i = hf; i < a.ss_count; i += TPR) v += pp[i];
#pragma unroll
      for (int off = 1; off < TPR; off <<= 1) v += __shfl_xor(v, off, 64);
      rs *= 1.0f / sqrtf(v / (float)a.K + a.eps);
    }
    if (hf == 0 && !same_rows) { s_xrow[r] = xrow; s_orow[r] = orow; s_rs[r] = rs; }
  }
  __syncthreads();

  S2D2_TTS(1);
  // ---- operand addressing ----
  const int c16 = tid & 7, rbase = tid >> 3;   // this thread stages rows rbase + (NTH / 8) i, bytes [16 c16, +16) of the 128
  // Loads in the K loop are unconditional (clamped addresses, values of invalid rows / columns replaced when
  // they are stored to LDS): a load under a branch would make the compiler wait for every outstanding load
  // before the MFMA block and so undo the weight pipeline.
  const bf16_t* xsrc[XI];
  bool xok[XI];
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int xr_ = s_xrow[rbase + (NTH / 8) * i];
    xok[i] = xr_ >= 0;
    xsrc[i] = a.X + (size_t)(xok[i] ? xr_ : 0) * a.ldx + c16 * 8;
  }
  const u32x4_t zero = {0u, 0u, 0u, 0u};

  f32x4_t acc[RBN][TN];
#pragma unroll
  for (int rb = 0; rb < RBN; ++rb)
#pragma unroll
    for (int t = 0; t < TN; ++t) acc[rb][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  u32x4_t xr[XD][XI], xl[XD][SPLIT ? XI : 1];
  constexpr int XL = XI * (SPLIT ? 2 : 1);   // activation loads per thread and step
  // One of the XL activation loads of a step: chunk j % XI of plane j / XI.  Unconditional: past the split's last
  // step the loads re-read an earlier tile into a register set nobody stores any more.
  // (plain: K is a multiple of the step, so the step's offset is the same for every lane)
  auto load_x1 = [&](u32x4_t (&r)[XI], u32x4_t (&l)[SPLIT ? XI : 1], int kb, int j, bool plain = false) __attribute__((always_inline)) {
    const int ko = plain ? min(kb, nk - 1) * TK
                         : min(min(kb, nk - 1) * TK + c16 * 8, a.K - 8) - c16 * 8;   // in bounds; columns at or past K are zeroed in store_x
    if (j < XI) r[j] = *(const u32x4_t*)(xsrc[j] + ko);
    else l[j - XI] = *(const u32x4_t*)(xsrc[j - XI] + a.x_lo + ko);
  };
  // (plain: every row of the tile is live and K is a multiple of the step: nothing to zero)
  auto store_x = [&](const u32x4_t (&r)[XI], const u32x4_t (&l)[SPLIT ? XI : 1], int buf, int kb, bool plain = false) __attribute__((always_inline)) {
    const bool kok = kb * TK + c16 * 8 < a.K;
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      const bool ok = plain || (xok[i] && kok);
      *(u32x4_t*)(s_xd + buf * XBUF + (rbase + (NTH / 8) * i) * XROW + c16 * 16) = ok ? r[i] : zero;
      if (SPLIT) *(u32x4_t*)(s_xd + buf * XBUF + (rbase + (NTH / 8) * i) * XROW + 128 + c16 * 16) = ok ? l[i] : zero;
    }
  };

  // Step j (counted from this split's first step) multiplies out of weight stage j % WS and LDS buffer j % 3.
  // The weights of step j + WS - 1 are requested during step j into the stage step j - 1 has just left.  The
  // activation tile of step j travels through register set j & 1: requested in the second half of step j - 4,
  // stored to LDS in the middle of step j - 2.  The workgroup's one barrier per step sits in the first quarter of
  // the step, ahead of that store.  So the store of step j (tile j + 2, into the buffer step j - 1 has read) comes
  // after a barrier every wavefront reached after its step j - 1, and the reads of tile j + 2, which begin at the
  // end of step j + 1, come after the barrier of step j + 1.  Nothing at a step's end waits for anything: the
  // operand reads run PD MFMA pairs ahead straight across the step boundary (an LDS read takes 130-250 clocks
  // here, an MFMA pair 32).  With two buffers, the store at the step's end and the barrier after it, every step
  // began with that latency on all eight wavefronts at once and ended with the wait for the stores: a third of
  // the step, measured with clock stamps per phase.
  // All memory requests are issued one at a time between the MFMA pairs: a burst of all of them at one place
  // keeps the address unit busy for as long as the MFMAs of the step take, with every wavefront of the
  // workgroup waiting in it at the same time.
#pragma unroll
  for (int d = 0; d < 2; ++d)
#pragma unroll
    for (int j = 0; j < XL; ++j) load_x1(xr[d], xl[d], kb0 + d, j);
  store_x(xr[0], xl[0], 0, kb0);
  store_x(xr[1], xl[1], 1, kb0 + 1);
#pragma unroll
  for (int d = 0; d < 2; ++d)
#pragma unroll
    for (int j = 0; j < XL; ++j) load_x1(xr[d], xl[d], kb0 + 2 + d, j);
  __syncthreads();
  S2D2_TTS(7);
  constexpr int UN = (WS % 3 ? 3 : 1) * (WS % 2 ? 2 : 1) * WS;   // unrolled steps: weight stage, register set and LDS buffer are compile-time
  constexpr int PL = SPLIT ? 2 : 1, NB = 2 * RBN * PL, PD = S2D2_TILE_PD;   // operand reads (= MFMA pairs) of a step; reads in flight
  constexpr int PB = 2, SB = RBN - 1;   // 16-row blocks (of 2 RBN) after which the barrier / the store come
  const uint8_t* xlds = s_xd + f * XROW + g * 16;
  auto xop = [&](int buf, int i) __attribute__((always_inline)) {   // operand of MFMA pair i of a step: K half, row block, plane
    const int k2 = i / (RBN * PL), rb = (i / PL) % RBN, pl = i % PL;
    return *(const u32x4_t*)(xlds + buf * XBUF + rb * 16 * XROW + pl * 128 + k2 * 64);
  };
  u32x4_t bq[PD];
#pragma unroll
  for (int i = 0; i < PD; ++i) bq[i] = xop(0, i);
#ifdef S2D2_KERNEL_TIMING
  unsigned long long step_sum[16] = {}, step_c = 0;
#endif
  // FULL: all UN steps exist.  The group that may end early is a second copy of the body: an exit out of the
  // unrolled body makes the compiler's wait-count bookkeeping drain every outstanding load in the first step of
  // each group (weights and activations requested for later steps included), and with it the weight pipeline.
  // ROWS: all 128 rows live and K a multiple of the step: no branches in the step, no zeroing of operands, and the
  // operand reads run ahead.
  auto group = [&](auto full_tag, auto rows_tag, int kbase) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_tag)::value, ROWS = decltype(rows_tag)::value;
#pragma unroll
    for (int u_ = 0; u_ < UN; ++u_) {
      const int st_ = u_ % WS, rs_ = (u_ + WS - 1) % WS;   // stage multiplied from, stage refilled
      const int kb = kbase + u_;
      if (!FULL && kb >= kb1) break;
      // what follows 16-row block blk of the step's 2 RBN: one of the 2 TN weight loads after every fourth block,
      // the barrier, the store of tile kb + 2, and after it the loads of tile kb + 4 into the same register set
      auto after_block = [&](int blk) __attribute__((always_inline)) {
        constexpr int WEVERY = 2 * RBN / (2 * TN);
        if (blk % WEVERY == 0) load_w1(wst[rs_][(blk / WEVERY) / TN][(blk / WEVERY) % TN], kb + WS - 1, (blk / WEVERY) / TN, (blk / WEVERY) % TN);
        // The barrier is the bare instruction: no wait for outstanding LDS traffic in front of it (the operand reads
        // in flight would have to drain, and the pipeline to refill, on all wavefronts at once).  None is needed: a
        // wavefront's LDS accesses complete in order, the store of the step before was followed by operand reads whose
        // values this wavefront has already multiplied, and so were its reads of the buffer the others overwrite next.
        // (The "memory" clobber keeps the compiler from moving LDS accesses across it.)
        if (blk == PB) asm volatile("s_barrier" ::: "memory");
        if (blk == SB && kb + 2 < kb1) store_x(xr[u_ & 1], xl[u_ & 1], (u_ + 2) % 3, kb + 2, ROWS);
#pragma unroll
        for (int j = 0; j < XL; ++j)
          if (SB + 1 + j * (2 * RBN - SB - 1) / XL == blk) load_x1(xr[u_ & 1], xl[u_ & 1], kb + 4, j, ROWS);
      };
      if (ROWS) {
        S2D2_STEP_CLK(0);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          const int k2 = i / (RBN * PL), rb = (i / PL) % RBN;
#pragma unroll
          for (int t = 0; t < TN; ++t)
            acc[rb][t] = mfma_16x16x32<OPM>(wst[st_][k2][t], bq[i % PD], acc[rb][t]);
          // (past the split's last step this reads some tile nobody multiplies)
          bq[i % PD] = i + PD < NB ? xop(u_ % 3, i + PD) : xop((u_ + 1) % 3, i + PD - NB);
          if (i % PL == PL - 1) after_block(i / PL);
          // (without this fence the instruction scheduler moves every read back down to right before its MFMA pair)
          __builtin_amdgcn_sched_barrier(0);
          if (S2D2_STEP_EIGHTHS && i % (NB / 8) == NB / 8 - 1) S2D2_STEP_CLK(1 + i / (NB / 8));
        }
      } else {
#pragma unroll
        for (int blk = 0; blk < 2 * RBN; ++blk) {
          const int k2 = blk / RBN, rb = blk % RBN;
          if (rb < rb_live) {   // else: 16-row block past the tile's rows
#pragma unroll
            for (int pl = 0; pl < PL; ++pl) {
              const u32x4_t b = xop(u_ % 3, blk * PL + pl);
#pragma unroll
              for (int t = 0; t < TN; ++t)
                acc[rb][t] = mfma_16x16x32<OPM>(wst[st_][k2][t], b, acc[rb][t]);
            }
          }
          after_block(blk);
        }
      }
    }
  };
  int kbase = kb0;
  if (rb_live == RBN && a.K % TK == 0) {
    for (; kbase + UN <= kb1; kbase += UN) group(std::true_type{}, std::true_type{}, kbase);
    if (kbase < kb1) group(std::false_type{}, std::true_type{}, kbase);
  } else {
    for (; kbase + UN <= kb1; kbase += UN) group(std::true_type{}, std::false_type{}, kbase);
    if (kbase < kb1) group(std::false_type{}, std::false_type{}, kbase);
  }

  if (acc[0][0][0] == 12345.678f) return true;
#ifdef S2D2_KERNEL_TIMING
  if (EPI == SEPI_SWIGLU && bx == 0 && ty == 0 && z == 0 && lane == 0)
    for (int k = 0; k < 16; ++k) g_tile_ts[896 + 16 * wave + k] = step_sum[k];
#endif
  S2D2_TTS(2);

  // ---- epilogue of one unit: v0 (and v1, the up projection, for SwiGLU) = accumulator(s) of row block rb, feature
  // tile nt0 + t of this wavefront: v[i] = Y[row wr*64 + rb*16 + f][feature (nt0 + t)*16 + 4 g + i].  rb and t may
  // be run-time values (the merge of a K split hands over sums it has just formed). ----
  auto epi_unit = [&](const int rb, const int t, const f32x4_t& v0, const f32x4_t& v1) __attribute__((always_inline)) {
    const int r = rb * 16 + f;
    const bool live = r < Mloc;
    const int orow = live ? s_orow[r] : 0;
    const float rs = s_rs[r];
    const int nt = nt0 + t;
    if (nt >= a.NT) return;   // uniform over the wavefront
    const int n = nt * 16 + 4 * g;
    if (EPI == SEPI_STORE_F32) {
      if (live) {
        float* op = (float*)a.out + (size_t)orow * a.ldo + n;
        const f32x4_t v = v0 * rs;
        if (n + 3 < a.N) *(float4*)op = make_float4(v[0], v[1], v[2], v[3]);
        else
          for (int i = 0; i < 4; ++i)
            if (n + i < a.N) op[i] = v[i];
      }
    } else if (EPI == SEPI_ADD_F32) {   // N is a multiple of 16 here: four features per lane as one 16-byte access
      float hv[4] = {0.f, 0.f, 0.f, 0.f};
      if (live) {
        float4* hp = (float4*)((float*)a.out + (size_t)orow * a.ldo + n);
        const float4 h0 = *hp;
        hv[0] = h0.x + v0[0] * rs;
        hv[1] = h0.y + v0[1] * rs;
        hv[2] = h0.z + v0[2] * rs;
        hv[3] = h0.w + v0[3] * rs;
        *hp = make_float4(hv[0], hv[1], hv[2], hv[3]);
        if (a.xg_out) {
          const float4 gn = *(const float4*)(a.gain_next + n);
          act_store4(a.xg_out + (size_t)orow * a.xg_ld + n, a.xg_lo, hv[0] * gn.x, hv[1] * gn.y, hv[2] * gn.z, hv[3] * gn.w);
        }
      }
      if (a.ss_out) {
        float sq = (hv[0] * hv[0] + hv[1] * hv[1]) + (hv[2] * hv[2] + hv[3] * hv[3]);
        sq += __shfl_xor(sq, 16, 64);
        sq += __shfl_xor(sq, 32, 64);
        if (live && g == 0) a.ss_out[(size_t)orow * a.ss_stride + nt] = sq;
      }
    } else if (EPI == SEPI_SWIGLU) {
      if (live) {
        float sv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float gate = v0[i] * rs, up = v1[i] * rs;
          sv[i] = gate / (1.0f + __expf(-gate)) * up;
        }
        act_store4((bf16_t*)a.out + (size_t)orow * a.ldo + n, a.out_lo, sv[0], sv[1], sv[2], sv[3]);
      }
    } else {  // SEPI_QKV_ROPE: features 0-7 of a tile pair with features 8-15 (lanes 32 apart)
      const int D = a.D, half = D >> 1, tiles_per_head = D / 16;
      const int head = nt / tiles_per_head, i0 = 8 * (nt % tiles_per_head) + 4 * (g & 1);
      float own[4], oth[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        own[i] = v0[i] * rs;
        oth[i] = __shfl_xor(own[i], 32, 64);
      }
      if (live) {
        const bool second = g >= 2;   // this lane holds x2 (element i + D/2) of the pair
        if (head < a.Hq + a.Hkv) {
          const bool is_q = head < a.Hq;
          bf16_t* dst = is_q ? a.q_out + (size_t)orow * a.q_ld + head * D
                             : a.k_out + ((size_t)orow * a.Hkv + (head - a.Hq)) * D;
          const float4 c01 = *(const float4*)(a.rope_cs + (size_t)orow * half + i0), c23 = *(const float4*)(a.rope_cs + (size_t)orow * half + i0 + 2);
          const float cs_c[4] = {c01.x, c01.z, c23.x, c23.z}, cs_s[4] = {c01.y, c01.w, c23.y, c23.w};
          float y[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) y[i] = second ? own[i] * cs_c[i] + oth[i] * cs_s[i] : own[i] * cs_c[i] - oth[i] * cs_s[i];
          // queries in the storage the attention kernel reads (q_lo); keys always as one bf16 plane (the cache's type)
          act_store4(dst + i0 + (second ? half : 0), is_q ? a.q_lo : 0, y[0], y[1], y[2], y[3]);
          if (!is_q && a.k16_out)   // the window's keys once more as half values (the attention kernel's copy)
            act_store4(a.k16_out + ((size_t)orow * a.Hkv + (head - a.Hq)) * D + i0 + (second ? half : 0), LO_F16, y[0], y[1], y[2], y[3]);
        } else {
          const int vh = head - a.Hq - a.Hkv;
          bf16_t* dst = a.v_out + ((size_t)orow * a.Hkv + vh) * D + (second ? half : 0);
          const int sq = a.row_seq[orow], tw = orow - a.seq_row0[sq];
          bf16_t b[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) b[i] = f32_to_bf16(own[i]);
          *(uint2*)(dst + i0) = make_uint2((uint32_t)b[0] | ((uint32_t)b[1] << 16), (uint32_t)b[2] | ((uint32_t)b[3] << 16));
          if (a.vT_out) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              a.vT_out[((size_t)(sq * a.Hkv + vh) * D + i0 + i + (second ? half : 0)) * a.wpad + tw] = a.win_f16 ? f32_to_f16_bits(own[i]) : b[i];
          }
        }
      }
    }
  };

  if (KS == 1) {
#pragma unroll
    for (int rb = 0; rb < RBN; ++rb)
#pragma unroll
      for (int t = 0; t < FT; ++t) epi_unit(rb, t, acc[rb][NACC * t], acc[rb][NACC == 2 ? 2 * t + 1 : 0]);
    __builtin_amdgcn_s_waitcnt(0);
    S2D2_TTS(6);
    return true;
  }

  // ---- split K ----
  // Partials in register order, [accumulator][half][thread] 8-byte words (every wavefront instruction covers 512
  // contiguous bytes), device-coherent write-through stores and loads around the tile's counter word (a
  // __threadfence pair per workgroup instead made the launches 60 % slower: the fences are cache-wide); 16-row
  // blocks past the tile's rows are neither written nor read.
  //
  // When the splits wait for each other (wait_ok), a split's own share never travels: the accumulators of units
  // z, z + KS, ... are parked in LDS behind the operand buffers (the merge addresses them with run-time unit numbers,
  // which registers cannot be) and only the other (KS - 1) / KS of the tile are written, and as much read back.  The
  // write-through partials are what the tail of a split launch consists of: from the slowest split's last K step to
  // "all partials there" 8-10 us with four splits and 17 us with eight (clock stamps of every workgroup), at 4 MB
  // per XCD and launch.  A split that gives its share up writes it out first.
  const size_t tile_id = (size_t)ty * ncol + bx;
  const bool keep_own = wait_ok && !SPLIT;   // (with two planes the operand buffers leave no room)
  constexpr int NU = RBN * FT;
  unsigned own_mask = 0;                      // units of this split's share
  if (keep_own)
    for (int u = z; u < NU; u += KS) own_mask |= 1u << u;
  uint64_t* mine = (uint64_t*)a.tile_partials + (tile_id * KS + z) * (32 * NTH) + tid;
  uint8_t* own_lds = s_xd + 3 * XBUF + wave * 8192 + lane * 16;   // [slot][lane] 16 bytes; slot = (index of the unit in the share) * NACC + accumulator
  auto store_partial = [&](int rb, int t, const f32x4_t& v) __attribute__((always_inline)) {
    __hip_atomic_store(mine + ((rb * TN + t) * 2) * NTH, (uint64_t)__float_as_uint(v[0]) | ((uint64_t)__float_as_uint(v[1]) << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(mine + ((rb * TN + t) * 2 + 1) * NTH, (uint64_t)__float_as_uint(v[2]) | ((uint64_t)__float_as_uint(v[3]) << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
#pragma unroll
  for (int rb = 0; rb < RBN; ++rb) {
    if (rb * 16 >= Mloc) continue;   // uniform over the wavefront
#pragma unroll
    for (int t = 0; t < TN; ++t) {
      const int u = rb * FT + t / NACC;
      if ((own_mask >> u) & 1) *(f32x4_t*)(own_lds + (__builtin_popcount(own_mask & ((1u << u) - 1)) * NACC + t % NACC) * 1024) = acc[rb][t];
      else store_partial(rb, t, acc[rb][t]);
    }
  }
  __builtin_amdgcn_s_waitcnt(0);   // write-through stores completed before the arrival is counted
  __syncthreads();
  // Counter word of the tile: bits 0-7 arrivals, bits 8-15 workgroups that are done with the word (the last of them
  // clears it for the next launch), bits 16-23 shares given up (bit 16 + z: split z will not finish its share).
  int* ctr = &a.tile_counters[tile_id];
  auto done_with_word = [&]() __attribute__((always_inline)) {
    const int done = __hip_atomic_fetch_add(ctr, 1 << 8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (((done >> 8) & 0xff) == KS - 1) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  if (tid == 0) {
    int share = 0;
    bool giving_up = false;
    const int prev = __hip_atomic_fetch_add(ctr, wait_ok ? 1 : 1 + (1 << (16 + z)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((prev & 0xff) == KS - 1) {
      share = (1 << z) | ((prev >> 16) & 0xff);   // the last arrival: its own share and every share given up so far
    } else if (wait_ok) {
      bool all = false;
      for (int spins = 0; spins < a.merge_spins && !all; ++spins) {
        __builtin_amdgcn_s_sleep(8);
        all = (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 0xff) == KS;
      }
      if (all) share = 1 << z;
      else giving_up = true;
    }
    if (!giving_up) done_with_word();
    s_share = giving_up ? -1 : share;
  }
  __syncthreads();
  if (s_share < 0) {   // (uniform) give the share up: write it out of its parking place, and only then say so
#pragma unroll
    for (int rb = 0; rb < RBN; ++rb) {
      if (rb * 16 >= Mloc) continue;
#pragma unroll
      for (int t = 0; t < TN; ++t) {
        const int u = rb * FT + t / NACC;
        if ((own_mask >> u) & 1)
          store_partial(rb, t, *(const f32x4_t*)(own_lds + (__builtin_popcount(own_mask & ((1u << u) - 1)) * NACC + t % NACC) * 1024));
      }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0) {   // if everybody has arrived in the meantime, nobody will take the share: keep it
      const bool all = (__hip_atomic_fetch_or(ctr, 1 << (16 + z), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & 0xff) == KS;
      done_with_word();
      s_share = all ? 1 << z : 0;
    }
    __syncthreads();
  }
  S2D2_TTS(3);
  const int share = s_share;
  if (!share) return true;
  S2D2_TTS(4);
  // Share zs = units zs, zs + KS, ... of every wavefront (a unit: one accumulator, for SwiGLU the gate / up pair).
  // The partials of all units of a share and of all splits are requested together (at most 128 registers) and
  // added in split order: one memory round trip per share.
  const uint64_t* src0 = (const uint64_t*)a.tile_partials + (tile_id * KS) * (32 * NTH) + tid;
  auto merge = [&](auto ksm_tag) __attribute__((always_inline)) {
    constexpr int KSM = decltype(ksm_tag)::value;   // KS <= KSM
    constexpr int BU = 32 / (NACC * KSM) < NU / 2 ? 32 / (NACC * KSM) : NU / 2;   // units per round: a whole share (at most NU / 2 units) within 128 registers
    for (int zs = 0; zs < KS; ++zs) {
      if (!((share >> zs) & 1)) continue;
      const bool parked = keep_own && zs == z;   // this split's own term waits in LDS
      int slot0 = 0;
      for (int u0 = zs; u0 < NU; u0 += KS * BU, slot0 += BU) {
        uint64_t v[BU][NACC][KSM][2];
#pragma unroll
        for (int j = 0; j < BU; ++j) {
          const int u = u0 + KS * j, rb = u / FT, t = u % FT;
          const bool ok = u < NU && rb * 16 < Mloc;   // uniform over the wavefront
#pragma unroll
          for (int c = 0; c < NACC; ++c)
#pragma unroll
            for (int zz = 0; zz < KSM; ++zz)
#pragma unroll
              for (int e = 0; e < 2; ++e)
                v[j][c][zz][e] = !(ok && zz < KS) ? 0ull
                                 : (parked && zz == z) ? *(const uint64_t*)(own_lds + ((slot0 + j) * NACC + c) * 1024 + e * 8)
                                 : __hip_atomic_load(src0 + (size_t)zz * (32 * NTH) + ((rb * TN + NACC * t + c) * 2 + e) * NTH,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int j = 0; j < BU; ++j) {
          const int u = u0 + KS * j, rb = u / FT, t = u % FT;
          if (u >= NU || rb * 16 >= Mloc) continue;   // uniform over the wavefront
          f32x4_t sum[NACC];
#pragma unroll
          for (int c = 0; c < NACC; ++c) {
            sum[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int zz = 0; zz < KSM; ++zz) {
              if (zz >= KS) break;   // uniform
              sum[c][0] += __uint_as_float((uint32_t)v[j][c][zz][0]);
              sum[c][1] += __uint_as_float((uint32_t)(v[j][c][zz][0] >> 32));
              sum[c][2] += __uint_as_float((uint32_t)v[j][c][zz][1]);
              sum[c][3] += __uint_as_float((uint32_t)(v[j][c][zz][1] >> 32));
            }
          }
          epi_unit(rb, t, sum[0], sum[NACC - 1]);
        }
      }
    }
  };
  if (KS <= 2) merge(std::integral_constant<int, 2>{});
  else if (KS <= 4) merge(std::integral_constant<int, 4>{});
  else merge(std::integral_constant<int, 8>{});
  __builtin_amdgcn_s_waitcnt(0);
  S2D2_TTS(6);
  return true;
}

// blockIdx.y = first row tile of the workgroup; it walks on in steps of gridDim.y while there are rows.
//
// Launches without a K split and with several row tiles (xcd_order: the host has padded gridDim.x to a multiple of
// 8) re-deal the tiles: the hardware hands consecutive workgroups to the 8 XCDs in turn, each with an L2 of its
// own, and with the plain order the row tiles of one column tile (which read the same weights) either sit on
// different XCDs or, on the same one, in different rounds of the launch; every column's weights then come in from
// memory once per row tile (measured: 2.2x the weight bytes for the verifier's gate / up projection of the 8 B
// model, 7.8x for the unembedding of 8 row tiles).  Here XCD i % 8 owns the column tiles c with c % 8 == i % 8 and
// takes them one after the other, all row tiles of a column next to each other in launch order.
template <int EPI, int PRO, int OPM, int WC>
__global__ __launch_bounds__(128 * WC, 2) void gemm_tile_kernel(const GemmStreamArgs a) {
  constexpr int COLS = (EPI == SEPI_SWIGLU ? 2 : 4) * WC;   // 16-feature tiles per workgroup
  // Three forms of the launch.  (1) plain: blockIdx = (column tile, first row tile, K split).  (2) xcd_order, see
  // above.  (3) stream_k (= row tiles of the launch): 3/2 tiles per workgroup.  A launch of 1.5 x as many tiles as
  // compute units otherwise runs two rounds, the second half empty; here every workgroup takes one tile whole and
  // then one half of K of a tile it shares with its neighbour on the XCD (workgroups w and w + 8), so both arrive at
  // the shared tile together and merge it as two splits.  Per XCD: its column tiles as in (2), tiles numbered row
  // tile fastest; its P workgroups take the first P tiles whole and the last P / 2 as halves, a workgroup's whole tile
  // and its half being of the same row tile, the pair of a shared tile being the workgroups of that row tile with
  // neighbouring whole columns.  Both parts are whole columns (the host checks that the row tiles divide P / 2), so
  // the weights of a column are read in one of the two phases only, by all its row tiles at the same time.  (With the shared tile taken out of the middle of every
  // three, each column's weights had left the XCD's L2 between the phases and came in from memory twice: 551 MB
  // fetched per launch of the 8 B model's gate / up projection against 201 MB of weights.)  In every form a
  // workgroup walks on over the row tiles past the expected ones (device-side row count above m_hint) as whole tiles.
  const int w = blockIdx.x, sk_rows = a.stream_k, sk_cols = (a.NT + COLS - 1) / COLS;
  int bx = blockIdx.x, by = blockIdx.y;
  if (a.xcd_order) {
    const int i = blockIdx.x + gridDim.x * blockIdx.y, s_ = i >> 3;
    bx = (s_ / (int)gridDim.y) * 8 + (i & 7);
    by = s_ % (int)gridDim.y;
    if (bx * COLS >= a.NT) return;   // padding of the grid
  }
  // (4) split_xcd: K splits dealt to XCDs.  In the plain order XCD i % 8 gets the column tiles c % 8 == i % 8 with all
  // their K splits, so every XCD reads all of the activation (for the 8 B model's down projection 8 x 12.6 MB, as
  // much as the weights).  Here XCD x takes split x % KS only, i.e. 1 / KS of the activation's columns, and among
  // the 8 / KS XCDs of a split each takes whole columns of tiles, all row tiles of a column next to each other.
  int bz = blockIdx.z;
  if (a.split_xcd) {
    const int i = blockIdx.x + (int)gridDim.x * (blockIdx.y + (int)gridDim.y * blockIdx.z), xcd = i & 7, s_ = i >> 3;
    const int KSg = gridDim.z, Q = 8 / KSg;
    bz = xcd % KSg;
    bx = (xcd / KSg) * ((int)gridDim.x / Q) + s_ / (int)gridDim.y;
    by = s_ % (int)gridDim.y;
  }
  const bool wait_ok = sk_rows > 0 || (long long)gridDim.x * gridDim.y * gridDim.z <= (long long)a.coop_wgs;
  bool did_prev = false;
  for (int it = 0;; ++it) {
    int tx = bx, ty = by + it * (int)gridDim.y, z = bz, ks = gridDim.z, ncol = gridDim.x;
    bool open_end = true;   // the items of this kind end with the first row tile that does not exist
    if (sk_rows > 0) {
      ncol = sk_cols; z = 0; ks = 1;
      if (it < 2) {
        // XCD w % 8 owns the column tiles c % 8 == w % 8; wl: this workgroup among the P of its XCD, cw: the columns
        // of its list that are taken whole.  Both items of a workgroup are of the same row tile, so the row maps
        // (and the sums behind 1/rms) of the first serve the second.
        const int wl = w >> 3, P = (int)gridDim.x >> 3, cw = P / sk_rows, q = wl / sk_rows;
        ty = wl % sk_rows;
        tx = (it == 0 ? q : cw + (q >> 1)) * 8 + (w & 7);
        open_end = false;
        if (it == 1) { z = q & 1; ks = 2; }
      } else {
        const int t = w + (it - 2) * (int)gridDim.x;
        tx = t % sk_cols; ty = sk_rows + t / sk_cols;
      }
    }
    const bool did = gemm_tile_body<EPI, PRO, OPM, WC>(a, tx, ty, z, ks, ncol, wait_ok, sk_rows > 0 && it == 1 && did_prev);
    did_prev = did;
    if (did) __syncthreads();   // the next tile reuses the LDS arrays
    else if (open_end) break;
  }
}

#ifdef S2D2_KERNEL_TIMING
__global__ void tile_ts_copy_kernel(unsigned long long* out) { for (int i = threadIdx.x; i < 1024; i += blockDim.x) out[i] = g_tile_ts[i]; }
void launch_tile_ts_copy(hipStream_t st, void* out) { S2D2_LAUNCH(tile_ts_copy_kernel, dim3(1), dim3(128), 0, st, (unsigned long long*)out); }
#else
void launch_tile_ts_copy(hipStream_t, void*) {}
#endif

template <int EPI, int PRO, int WC>
static void launch_tile(hipStream_t st, const GemmStreamArgs& a, int row_tiles) {
  constexpr int COLS = (EPI == SEPI_SWIGLU ? 2 : 4) * WC;   // 16-feature tiles per workgroup
  constexpr int RESIDENT = WC == 2 ? 512 : 256;             // workgroups of one round over the chip
  constexpr double PART_BYTES = 32768.0 * WC;                // fp32 partial of one tile and split
  const int col_tiles = (a.NT + COLS - 1) / COLS;
  // K is split over blockIdx.z when that shortens the launch.  The choice minimises a small cost model fitted to
  // kernel traces of the batched configurations (microseconds; a round is as many workgroups as are resident on
  // the chip at once):
  //   rounds * (K steps per split * 1.05 + 6)                       K loop + prologue / epilogue per round
  //   + [splits > 1] * 10                                           partial write, wait and shared merge, or, when the
  //     launch has more workgroups than compute units (nobody waits, the last arrival merges the tile):
  //     8 + live tiles * splits * partial bytes * 2 / 3 TB/s
  // It is judged on the rows the caller expects (m_hint).  Every split keeps at least 4 K steps and the partials
  // must fit their buffer.
  int KS = 1;
  const long long tiles = (long long)col_tiles * row_tiles;
  const int hint_tiles = a.m_hint > 0 ? std::min(row_tiles, (a.m_hint + TM - 1) / TM) : row_tiles;
  const long long live = (long long)col_tiles * hint_tiles;
  const int nk = (a.K + TK - 1) / TK;
  const double step_us = 1.05, merge_us = 10.0, round_us = 6.0;
  if (a.tile_partials && a.grouped == GROUP_NONE && tiles <= a.tile_counter_cap) {
    double best = 1e30;
    for (int ks = 1; ks <= 8; ++ks) {
      if (ks > 1 && (nk / ks < 4 || tiles * ks * (WC / 2) > a.tile_partial_cap)) break;
      const double rounds = (double)((live * ks + RESIDENT - 1) / RESIDENT), steps = (double)((nk + ks - 1) / ks);
      double t = rounds * (steps * step_us + round_us);
      if (ks > 1) t += live * ks <= a.coop_wgs ? merge_us : 8.0 + (double)live * ks * PART_BYTES * 2.0 / 3.0e6;
      if (t < best - 1e-9) { best = t; KS = ks; }
    }
  }
  // blockIdx.y: the row tiles the caller expects (a workgroup walks on if there are more); all of them for the
  // expert-grouped launches, whose tile list lives on the device
  dim3 grid(col_tiles, a.grouped == GROUP_NONE ? hint_tiles : row_tiles, KS), block(128 * WC);
  GemmStreamArgs b = a;
  const char* sp = getenv("S2D2_TILE_SPINS");   // test aid: 0 makes every split give its share up at once (the hand-over path)
  b.merge_spins = sp ? atoi(sp) : 96;            // polls of about 1 us each
  b.xcd_order = a.grouped == GROUP_NONE && KS == 1 && grid.y > 1;
  b.stream_k = 0;
  // K splits dealt to XCDs (see the kernel): splits that divide the 8 XCDs, whole columns of tiles per XCD
  b.split_xcd = a.grouped == GROUP_NONE && KS > 1 && 8 % KS == 0 && col_tiles % (8 / KS) == 0 &&
                ((long long)col_tiles * hint_tiles * KS) % 8 == 0;
  if (b.xcd_order && WC == 4 && a.tile_partials && a.coop_wgs > 0 && 2 * live == 3LL * a.coop_wgs && (a.coop_wgs & 15) == 0 && (col_tiles & 7) == 0 && (a.coop_wgs / 16) % hint_tiles == 0 &&
      live <= a.tile_counter_cap && live * 2 * (WC / 2) <= a.tile_partial_cap && nk >= 8) {
    b.stream_k = hint_tiles;   // see the kernel: 3/2 tiles per workgroup, one workgroup per compute unit
    b.xcd_order = 0;
    grid = dim3(a.coop_wgs, 1, 1);
  }
  if (b.xcd_order) grid.x = (grid.x + 7) / 8 * 8;
  const int opm = operand_mode(a.x_lo);
  // three activation tiles in LDS (54 KB; 102 KB with two planes, above the 64 KB a kernel gets without asking)
  // (one plane: plus 8 KB per wavefront in which a K split parks its own share of the accumulators)
  const unsigned lds = 3u * TM * ((opm == OPM_BF16X2 ? 256 : 128) + 16) + (opm == OPM_BF16X2 ? 0u : 2u * WC * 8192u);
  static bool lds_set[3][64];
  const int oi = opm == OPM_F16 ? 0 : opm == OPM_BF16X2 ? 1 : 2;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) dev = -1;
  if (dev >= 0 && dev < 64 && !lds_set[oi][dev]) {
    const void* fn = opm == OPM_F16      ? (const void*)gemm_tile_kernel<EPI, PRO, OPM_F16, WC>
                     : opm == OPM_BF16X2 ? (const void*)gemm_tile_kernel<EPI, PRO, OPM_BF16X2, WC>
                                         : (const void*)gemm_tile_kernel<EPI, PRO, OPM_BF16, WC>;
    // on failure the launch below fails too, and the entry point reports that error
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess) lds_set[oi][dev] = true;
  }
  if (opm == OPM_F16) S2D2_LAUNCH((gemm_tile_kernel<EPI, PRO, OPM_F16, WC>), grid, block, lds, st, b);
  else if (opm == OPM_BF16X2) S2D2_LAUNCH((gemm_tile_kernel<EPI, PRO, OPM_BF16X2, WC>), grid, block, lds, st, b);
  else S2D2_LAUNCH((gemm_tile_kernel<EPI, PRO, OPM_BF16, WC>), grid, block, lds, st, b);
}

template <int EPI, int PRO>
static void launch_tile(hipStream_t st, const GemmStreamArgs& a, int row_tiles) {
  const char* e = getenv("S2D2_TILE_WC");   // tuning aid, read per launch so that a test can cover both shapes
  const int wc = e ? atoi(e) : 4;
  if (wc == 4) launch_tile<EPI, PRO, 4>(st, a, row_tiles);
  else launch_tile<EPI, PRO, 2>(st, a, row_tiles);
}

// row_tiles: upper bound of 128-row tiles (ungrouped: ceil(m_cap / 128); grouped: capacity of the tile list)
void launch_gemm_tile(hipStream_t st, int kind, int pro, const GemmStreamArgs& a, int row_tiles) {
  switch (kind) {
    case SEPI_QKV_ROPE: launch_tile<SEPI_QKV_ROPE, SPRO_BF16S>(st, a, row_tiles); break;
    case SEPI_ADD_F32: launch_tile<SEPI_ADD_F32, SPRO_BF16>(st, a, row_tiles); break;
    case SEPI_SWIGLU: launch_tile<SEPI_SWIGLU, SPRO_BF16S>(st, a, row_tiles); break;
    case SEPI_STORE_F32:
      if (pro == SPRO_BF16S) launch_tile<SEPI_STORE_F32, SPRO_BF16S>(st, a, row_tiles);
      else launch_tile<SEPI_STORE_F32, SPRO_BF16>(st, a, row_tiles);
      break;
  }
}

}  // namespace s2d2
