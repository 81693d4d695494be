// Whole decoder forward in ONE persistent launch, for windows of at most 16 rows (batch-1 style decoding).
//
// With a handful of window rows every layer is five short dependent phases (QKV + RoPE, attention,
// O projection, gate/up + SwiGLU, down projection) that each move only 1-50 MB: as separate kernels
// they are dominated by launch, ramp-up and drain rather than by HBM bandwidth.  Here one workgroup per
// compute unit stays resident for the whole forward; phases are separated by a device-wide barrier
// (arrival counters in 8 groups plus a top counter, bounded spin), and before a workgroup waits at a
// barrier it issues the loads of the first weight fragments of its NEXT phase, which depend on nothing,
// so HBM keeps streaming while the barrier resolves.
//
// Data that one phase hands to the next is written with device-coherent write-through stores
// (s2d2_internal.h); a producer waits for its stores before it arrives at the barrier.  No cache-wide
// fence is used.  What only the few attention workgroups read (q, window K / V) is read with
// device-coherent loads.  What every workgroup reads (the operand planes of the GEMMs, the attention
// output, the partial sums of squares) is read with ordinary cached loads, which is safe because
//   * every layer has its own buffers, so within a launch an address is written once and only read
//     after the barrier that follows its production: no L2 can hold an older copy of it, and
//   * the planes are tile-blocked: the 16 rows x 16 features a producer workgroup writes are 512
//     contiguous bytes, so no cache line has two writers.
// The residual stream never leaves the chip: the workgroup that owns 16 output features of the O /
// down projections keeps its 16 x 16 fp32 tile of h in LDS across layers.
//
// GEMM phases reuse the decomposition of the streaming kernel (packed 16 x 32 weight tiles as MFMA A
// operands, the 8 wavefronts of a workgroup split K, fixed-order merge through LDS, same fused
// epilogues); attention is the flash body of attention_flash.h.  Results do not depend on timing.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"
#include "attention_flash.h"

#include <algorithm>

namespace s2d2 {

static constexpr int FW = 8;      // wavefronts per workgroup
static constexpr int FU = 8;      // weight fragments per wavefront per batch
#ifdef S2D2_FUSED_TIMING
__device__ unsigned long long* g_ts = nullptr;
__device__ __forceinline__ void inner_stamp(int k) {
  if (threadIdx.x == 0 && blockIdx.x == gridDim.x - 1 && g_ts) g_ts[k] = wall_clock64();
}
#else
__device__ __forceinline__ void inner_stamp(int) {}
#endif

// The thread index behind an empty asm: address arithmetic derived from it is recomputed where it is used
// instead of being hoisted out of the layer loop and kept in registers across every phase.
__device__ __forceinline__ int opaque_tid() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}

__device__ __forceinline__ bool grid_sync(const FusedArgs& a, uint32_t epoch, int* s_ok) {
  __builtin_amdgcn_s_waitcnt(0);  // this wavefront's coherent stores have completed
  __syncthreads();
  if (threadIdx.x == 0) {
    const int G = gridDim.x, grp = blockIdx.x & 7, gsz = (G - grp + 7) >> 3;
    uint32_t* gc = a.bar + 64 * (1 + grp);
    const uint32_t prev = __hip_atomic_fetch_add(gc, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (prev == epoch * gsz + gsz - 1) __hip_atomic_fetch_add(a.bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int ok = 1, spins = 0;
    while (__hip_atomic_load(a.bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (epoch + 1) * 8u) {
      if (++spins > a.spin_limit) {  // some workgroup never arrived (not co-resident, or it gave up): poison and leave
        ok = 0;
        __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    *s_ok = ok;
  }
  __syncthreads();
  return *s_ok != 0;
}

// Loads through a uniform base pointer plus a 32-bit per-lane byte offset (one address register per phase
// instead of one 64-bit pointer per unrolled load).
__device__ __forceinline__ u32x4_t ldw(const uint4* base, uint32_t byte_off) {
  return *(const u32x4_t*)((const char*)base + byte_off);
}
__device__ __forceinline__ u32x4_t ldx(const bf16_t* base, uint32_t byte_off) {
  return *(const u32x4_t*)((const char*)base + byte_off);
}

// First batch of weight fragments (matrix 0) of tile nt for this wavefront's share of K.
__device__ __forceinline__ void prefetch_w(u32x4_t (&wpre)[FU], const uint4* Wp, int KT, int nt) {
  const int tq = opaque_tid();
  const int lane = tq & 63, wave = tq >> 6;
  const int kt_begin = (int)((long long)wave * KT / FW), kt_end = (int)((long long)(wave + 1) * KT / FW);
  const uint32_t off = (uint32_t)(((nt * KT + kt_begin) * 64 + lane) * 16);
  const u32x4_t zero = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int u = 0; u < FU; ++u) wpre[u] = (kt_begin + u < kt_end) ? ldw(Wp, off + u * 1024) : zero;
}

// 1 / rms of a window row from the per-tile partial sums of squares ([tile][32] floats: one cache line per
// producer).  The loads are issued at the start of a phase together with the operand loads and summed after
// the MFMA work: thread (row, sub) of threads < 256 holds every 16th partial, the 16 lanes of a row add up.
static constexpr int SSV = 16;   // d <= 4096
__device__ __forceinline__ void ss_issue(const float* ss, int NTd, int M, int tq, float (&sv)[SSV]) {
  const int row = tq >> 4, sub = tq & 15;
#pragma unroll
  for (int j = 0; j < SSV; ++j) {
    const int i = sub + 16 * j;
    sv[j] = (tq < 256 && row < M && i < NTd) ? ss[i * 32 + row] : 0.f;
  }
}
__device__ __forceinline__ float ss_finish(const float (&sv)[SSV], int d, float eps) {
  float v = 0.f;
#pragma unroll
  for (int j = 0; j < SSV; ++j) v += sv[j];
  v += __shfl_xor(v, 1, 64);
  v += __shfl_xor(v, 2, 64);
  v += __shfl_xor(v, 4, 64);
  v += __shfl_xor(v, 8, 64);
  return 1.0f / sqrtf(v / (float)d + eps);
}

enum { FEPI_QKV = 0, FEPI_ADD = 1, FEPI_SWIGLU = 2 };

// One batch of up to FU k-tiles: activation fragments (both planes; they are the dependent loads, so they go
// first), weight fragments (matrix 0 from the prefetched registers if USEPRE).  woff / xoff: byte offsets of
// this lane's fragment of k-tile kt0 in the weight matrix / the activation plane; XS: bytes per k-tile in X.
template <int NACC, bool USEPRE, int XS>
__device__ __forceinline__ void mac_batch(f32x4_t (&acc)[NACC], const uint4* W0, const uint4* W1, const bf16_t* X,
                                          uint32_t woff, uint32_t xoff, uint32_t xlo_bytes, bool row_ok, int kt0, int kt_end,
                                          const u32x4_t (&wpre)[FU]) {
  const u32x4_t zero = {0u, 0u, 0u, 0u};
  u32x4_t xh[FU], xl[FU], w0[USEPRE ? 1 : FU], w1[NACC == 2 ? FU : 1];
#pragma unroll
  for (int u = 0; u < FU; ++u) {
    const bool ok = row_ok && kt0 + u < kt_end;
    xh[u] = ok ? ldx(X, xoff + u * XS) : zero;
    xl[u] = ok ? ldx(X, xoff + xlo_bytes + u * XS) : zero;
  }
#pragma unroll
  for (int u = 0; u < FU; ++u) {
    const bool ok = kt0 + u < kt_end;
    if (!USEPRE) w0[u] = ok ? ldw(W0, woff + u * 1024) : zero;
    if (NACC == 2) w1[u] = ok ? ldw(W1, woff + u * 1024) : zero;
  }
#pragma unroll
  for (int u = 0; u < FU; ++u) {
    const bf16x8_t wa = __builtin_bit_cast(bf16x8_t, USEPRE ? wpre[u] : w0[USEPRE ? 0 : u]);
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8_t, xh[u]), acc[0], 0, 0, 0);
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8_t, xl[u]), acc[0], 0, 0, 0);
    if (NACC == 2) {
      const bf16x8_t wb = __builtin_bit_cast(bf16x8_t, w1[NACC == 2 ? u : 0]);
      acc[NACC - 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, __builtin_bit_cast(bf16x8_t, xh[u]), acc[NACC - 1], 0, 0, 0);
      acc[NACC - 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, __builtin_bit_cast(bf16x8_t, xl[u]), acc[NACC - 1], 0, 0, 0);
    }
  }
}

// One 16-feature tile: Y[m, nt*16 + f] = sum_k X[m, k] W[nt*16 + f, k] over both activation planes.
// PRE: wpre holds the first batch of matrix 0.  BLOCKED: X is a tile-blocked plane (element (row, n) at
// ((n >> 4) * 16 + row) * 16 + (n & 15), low plane xlo_bytes further on); else row-major with ldx elements
// per row.  On return threads < 256 (row = tid / 16, fe = tid % 16) hold the totals of their (row, feature):
// tot0 / tot1 for the two matrices, tot0b / tot1b for feature fe ^ 8.
template <int NACC, bool PRE, bool BLOCKED>
__device__ __forceinline__ void tile_mac(const uint4* Wp, const uint4* Wp2, int KT, int nt, int M, const bf16_t* X, int ldx,
                                         uint32_t xlo_bytes, const u32x4_t (&wpre)[FU], float* s_red, float& tot0,
                                         float& tot1, float& tot0b, float& tot1b) {
  constexpr int XS = BLOCKED ? 1024 : 64;
  const int tq = opaque_tid();
  const int lane = tq & 63, wave = tq >> 6;
  const int g = lane >> 4, f = lane & 15;
  const int kt_begin = (int)((long long)wave * KT / FW), kt_end = (int)((long long)(wave + 1) * KT / FW);
  const bool row_ok = f < M;
  uint32_t woff = (uint32_t)(((nt * KT + kt_begin) * 64 + lane) * 16);
  const int fr = row_ok ? f : 0;
  uint32_t xoff = BLOCKED ? (uint32_t)(kt_begin * 1024 + (g >> 1) * 512 + fr * 32 + (g & 1) * 16)
                          : (uint32_t)((fr * ldx + g * 8 + kt_begin * 32) * 2);
  f32x4_t acc[NACC];
#pragma unroll
  for (int t = 0; t < NACC; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  inner_stamp(0);
  mac_batch<NACC, PRE, XS>(acc, Wp, Wp2, X, woff, xoff, xlo_bytes, row_ok, kt_begin, kt_end, wpre);
  if (acc[0][0] == 12345.678f) inner_stamp(9);   // forces the first batch to complete before the next stamp
  inner_stamp(1);
  for (int kt0 = kt_begin + FU; kt0 < kt_end; kt0 += FU) {
    woff += FU * 1024;
    xoff += FU * XS;
    mac_batch<NACC, false, XS>(acc, Wp, Wp2, X, woff, xoff, xlo_bytes, row_ok, kt0, kt_end, wpre);
  }
  // acc[t][i] = Y[row f][feature 4 g + i]; merge the wavefronts in a fixed order
#pragma unroll
  for (int t = 0; t < NACC; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) s_red[((size_t)wave * NACC + t) * 256 + i * 64 + lane] = acc[t][i];
  inner_stamp(2);
  __syncthreads();
  inner_stamp(3);
  tot0 = tot1 = tot0b = tot1b = 0.f;
  if (tq < 256) {
    const int row = tq >> 4, fe = tq & 15;
    const int src = (fe & 3) * 64 + (fe >> 2) * 16 + row;
    const int fb = fe ^ 8, srcb = (fb & 3) * 64 + (fb >> 2) * 16 + row;   // partner feature (RoPE pairs)
#pragma unroll
    for (int w_ = 0; w_ < FW; ++w_) {
      tot0 += s_red[((size_t)w_ * NACC) * 256 + src];
      tot0b += s_red[((size_t)w_ * NACC) * 256 + srcb];
      if (NACC == 2) {
        tot1 += s_red[((size_t)w_ * NACC + 1) * 256 + src];
        tot1b += s_red[((size_t)w_ * NACC + 1) * 256 + srcb];
      }
    }
  }
  __syncthreads();   // s_red may be rewritten by the next tile
  inner_stamp(4);
}

// Operand v of threads (row, fe) of one producer tile into the tile-blocked planes: four features per 8-byte
// write-through store.  Every thread of the 16-lane row group calls it (shuffles); `live` rows are stored.
__device__ __forceinline__ void store_block(bf16_t* hi_plane, bf16_t* lo_plane, int tile, int row, int fe, float v, bool live) {
  bf16_t hi, lo;
  split_bf16(v, hi, lo);
  uint32_t ph = (uint32_t)hi | ((uint32_t)__shfl_down((int)hi, 1, 64) << 16);
  uint32_t pl = (uint32_t)lo | ((uint32_t)__shfl_down((int)lo, 1, 64) << 16);
  const uint32_t ph2 = (uint32_t)__shfl_down((int)ph, 2, 64), pl2 = (uint32_t)__shfl_down((int)pl, 2, 64);
  if (live && (fe & 3) == 0) {
    const size_t e = ((size_t)tile * 16 + row) * 16 + fe;
    st8_coh(hi_plane + e, make_uint2(ph, ph2));
    st8_coh(lo_plane + e, make_uint2(pl, pl2));
  }
}

__global__ __launch_bounds__(FW * 64) void forward_fused_kernel(const FusedArgs a) {
  extern __shared__ float smem[];          // attention merge slots / GEMM merge area
  __shared__ float s_h[16 * 16];           // this workgroup's tile of the residual stream (owners only)
  __shared__ int s_ok;
  const int G = gridDim.x, wg = blockIdx.x, tid = threadIdx.x;
  if (__hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;   // poisoned by an earlier failure
  const int M = min(16, a.plan.counts[0]);
  const int d = a.d, NTd = d >> 4, HqD = a.Hq * a.D, qkv_n = (a.Hq + 2 * a.Hkv) * a.D;
  const int NT1 = qkv_n >> 4, NT4 = a.F >> 4;
  const int KTd = d >> 5, KTo = HqD >> 5, KTf = a.F >> 5;
  const int owner_tile = wg - (G - NTd);                 // >= 0: owner of residual features [16 owner_tile, +16)
  const bool is_owner = owner_tile >= 0;
  const int n_attn = a.n_seq * a.Hkv * a.Z;
  const bool is_attn = wg < n_attn;
  const int ld_a = 2 * d, lo_a = d, ld_o = 2 * HqD, lo_o = HqD;
  // per-layer exchange buffers (bytes): xgA hi|lo, xgB hi|lo, ffn hi|lo, o, ssA, ssB
  const size_t pl_d = (size_t)NTd * 512, pl_f = (size_t)NT4 * 512, o_bytes = (size_t)16 * ld_o * 2, ss_bytes = (size_t)NTd * 128;
  uint32_t epoch = 0;
#ifdef S2D2_FUSED_TIMING
  int tslot = 0;
#define S2D2_STAMP() do { if (tid == 0 && (wg == 0 || wg == G - 1) && tslot < 400) a.tstamp[(wg ? 400 : 0) + tslot++] = wall_clock64(); } while (0)
#else
#define S2D2_STAMP() do {} while (0)
#endif
#define S2D2_ROLE                                   /* epilogue role of threads < 256, recomputed per phase */ \
  const int tq = opaque_tid();                                                                              \
  const int row = tq >> 4, fe = tq & 15;                                                                    \
  const bool live = tq < 256 && row < M;
  u32x4_t wpre[FU];
  float t0, t1, t0b, t1b;
#ifdef S2D2_FUSED_TIMING
  if (tid == 0 && wg == G - 1) g_ts = a.tstamp + 790;
#endif

  // ---- phase 0: embedding rows into the residual tile, operand and partial sums of the first norm ----
  prefetch_w(wpre, a.layers[0].wqkv, KTd, min(wg, NT1 - 1));
  if (is_owner && tid < 256) {
    S2D2_ROLE
    const int n = owner_tile * 16 + fe;
    float hv = 0.f;
    if (live) hv = bf16_to_f32(a.embed[(size_t)a.plan.row_token[row] * d + n]);
    s_h[row * 16 + fe] = hv;
    float sq = hv * hv;
    sq += __shfl_xor(sq, 1, 64);
    sq += __shfl_xor(sq, 2, 64);
    sq += __shfl_xor(sq, 4, 64);
    sq += __shfl_xor(sq, 8, 64);
    bf16_t* xg0 = (bf16_t*)a.act;
    store_block(xg0, xg0 + pl_d / 2, owner_tile, row, fe, hv * a.layers[0].norm1[n], live);
    if (live && fe == 0) st4f_coh((float*)(a.act + 4 * pl_d + 2 * pl_f + o_bytes) + owner_tile * 32 + row, sq);
  }

  for (int l = 0; l < a.n_layers; ++l) {
    const FusedLayer& L = a.layers[l];
    char* act = a.act + (size_t)l * a.act_stride;
    bf16_t* xgA = (bf16_t*)act;
    bf16_t* xgB = (bf16_t*)(act + 2 * pl_d);
    bf16_t* ffn = (bf16_t*)(act + 4 * pl_d);
    bf16_t* obuf = (bf16_t*)(act + 4 * pl_d + 2 * pl_f);
    float* ssA = (float*)(act + 4 * pl_d + 2 * pl_f + o_bytes);
    float* ssB = (float*)(act + 4 * pl_d + 2 * pl_f + o_bytes + ss_bytes);
    char* act_next = act + a.act_stride;
    bf16_t* xgA_next = (bf16_t*)act_next;
    float* ssA_next = (float*)(act_next + 4 * pl_d + 2 * pl_f + o_bytes);
    bf16_t* kw = a.k_stage + (size_t)l * a.stage_layer;
    bf16_t* vw = a.v_stage + (size_t)l * a.stage_layer;
    S2D2_STAMP();
    if (!grid_sync(a, epoch++, &s_ok)) return;
    S2D2_STAMP();

    // ---- phase 1: QKV projection, RoPE, q / k / v split ----
    float sv[SSV], rs = 0.f;
    ss_issue(ssA, NTd, M, opaque_tid(), sv);
    for (int nt = wg; nt < NT1; nt += G) {
      if (nt == wg) tile_mac<1, true, true>(L.wqkv, nullptr, KTd, nt, M, xgA, 0, (uint32_t)pl_d, wpre, smem, t0, t1, t0b, t1b);
      else tile_mac<1, false, true>(L.wqkv, nullptr, KTd, nt, M, xgA, 0, (uint32_t)pl_d, wpre, smem, t0, t1, t0b, t1b);
      S2D2_ROLE
      if (nt == wg && tq < 256) rs = ss_finish(sv, d, a.eps);
      if (live && fe < 8) {   // lanes fe < 8 own the rotation pair (i, i + D/2) of one head
        const int D = a.D, half = D >> 1, tiles_per_head = D >> 4;
        const int head = nt / tiles_per_head, i = 8 * (nt % tiles_per_head) + fe;
        const float x1 = t0 * rs, x2 = t0b * rs;
        if (head < a.Hq + a.Hkv) {
          const float2 cs = a.rope_cs[(size_t)row * half + i];
          const float y1 = x1 * cs.x - x2 * cs.y, y2 = x2 * cs.x + x1 * cs.y;
          if (head < a.Hq) {
            bf16_t* dst = a.q + (size_t)row * ld_o + head * D;
            bf16_t h1, l1, h2, l2;
            split_bf16(y1, h1, l1);
            split_bf16(y2, h2, l2);
            st2_coh(dst + i, h1);
            st2_coh(dst + i + half, h2);
            st2_coh(dst + lo_o + i, l1);
            st2_coh(dst + lo_o + i + half, l2);
          } else {
            bf16_t* dst = kw + ((size_t)row * a.Hkv + (head - a.Hq)) * D;
            st2_coh(dst + i, f32_to_bf16(y1));
            st2_coh(dst + i + half, f32_to_bf16(y2));
          }
        } else {
          const int vh = head - a.Hq - a.Hkv;
          const bf16_t b1 = f32_to_bf16(x1), b2 = f32_to_bf16(x2);
          bf16_t* dst = vw + ((size_t)row * a.Hkv + vh) * D;
          st2_coh(dst + i, b1);
          st2_coh(dst + i + half, b2);
          const int sq = a.plan.row_seq[row], tw = row - a.plan.seq_row0[sq];
          bf16_t* vt = a.vT_win + ((size_t)(sq * a.Hkv + vh) * D) * a.wpad + tw;
          st2_coh(vt + (size_t)i * a.wpad, b1);
          st2_coh(vt + (size_t)(i + half) * a.wpad, b2);
        }
      }
    }
    if (!is_attn) {  // attention workgroups fetch after their attention phase: its registers are all in use
      if (is_owner) prefetch_w(wpre, L.wo, KTo, owner_tile);
      else prefetch_w(wpre, L.wg, KTd, min(wg, NT4 - 1));
    }
    S2D2_STAMP();
    if (!grid_sync(a, epoch++, &s_ok)) return;
    S2D2_STAMP();

    // ---- phase 2: attention over the paged prefix cache and the window ----
    if (is_attn) {
      const size_t part_ml_off = (size_t)n_attn * 32 * FA_D;
      attn_flash_body<FW, true, true>(a.q, ld_o, lo_o, kw, a.vT_win, a.k_pages + (size_t)l * a.page_layer,
                                      a.v_pages + (size_t)l * a.page_layer, a.g, a.plan, a.Hq, a.Z, a.wpad, a.scale_log2e,
                                      obuf, ld_o, lo_o, a.part, a.part + part_ml_off, a.attn_counters, wg % a.Z, 0, wg / a.Z, 1,
                                      smem);
      __syncthreads();
      if (is_owner) prefetch_w(wpre, L.wo, KTo, owner_tile);
      else prefetch_w(wpre, L.wg, KTd, min(wg, NT4 - 1));
    }
    S2D2_STAMP();
    if (!grid_sync(a, epoch++, &s_ok)) return;
    S2D2_STAMP();

    // ---- phase 3: O projection, residual add, operand and partial sums of the second norm ----
    if (is_owner) {
      const float gn = L.norm2[owner_tile * 16 + (opaque_tid() & 15)];   // issued before the operand loads
      tile_mac<1, true, false>(L.wo, nullptr, KTo, owner_tile, M, obuf, ld_o, (uint32_t)lo_o * 2, wpre, smem, t0, t1, t0b, t1b);
      S2D2_ROLE
      if (tq < 256) {
        float hv = 0.f;
        if (live) { hv = s_h[row * 16 + fe] + t0; s_h[row * 16 + fe] = hv; }
        float sq = hv * hv;
        sq += __shfl_xor(sq, 1, 64);
        sq += __shfl_xor(sq, 2, 64);
        sq += __shfl_xor(sq, 4, 64);
        sq += __shfl_xor(sq, 8, 64);
        store_block(xgB, xgB + pl_d / 2, owner_tile, row, fe, hv * gn, live);
        if (live && fe == 0) st4f_coh(ssB + owner_tile * 32 + row, sq);
      }
      prefetch_w(wpre, L.wg, KTd, min(wg, NT4 - 1));
    }
    S2D2_STAMP();
    if (!grid_sync(a, epoch++, &s_ok)) return;
    S2D2_STAMP();

    // ---- phase 4: gate / up projections and SwiGLU ----
    ss_issue(ssB, NTd, M, opaque_tid(), sv);
    for (int nt = wg; nt < NT4; nt += G) {
      if (nt == wg) tile_mac<2, true, true>(L.wg, L.wu, KTd, nt, M, xgB, 0, (uint32_t)pl_d, wpre, smem, t0, t1, t0b, t1b);
      else tile_mac<2, false, true>(L.wg, L.wu, KTd, nt, M, xgB, 0, (uint32_t)pl_d, wpre, smem, t0, t1, t0b, t1b);
      S2D2_ROLE
      if (nt == wg && tq < 256) rs = ss_finish(sv, d, a.eps);
      if (tq < 256) {
        const float gate = t0 * rs, up = t1 * rs;
        store_block(ffn, ffn + pl_f / 2, nt, row, fe, gate / (1.0f + __expf(-gate)) * up, live);
      }
    }
    const bool more = l + 1 < a.n_layers;
    if (is_owner) prefetch_w(wpre, L.wdown, KTf, owner_tile);
    else if (more) prefetch_w(wpre, a.layers[l + 1].wqkv, KTd, min(wg, NT1 - 1));
    S2D2_STAMP();
    if (!grid_sync(a, epoch++, &s_ok)) return;
    S2D2_STAMP();

    // ---- phase 5: down projection, residual add, operand and partial sums of the next norm ----
    if (is_owner) {
      const float* gain_next = more ? a.layers[l + 1].norm1 : a.norm_f;
      const float gn = gain_next[owner_tile * 16 + (opaque_tid() & 15)];
      tile_mac<1, true, true>(L.wdown, nullptr, KTf, owner_tile, M, ffn, 0, (uint32_t)pl_f, wpre, smem, t0, t1, t0b, t1b);
      S2D2_ROLE
      if (tq < 256) {
        const int n = owner_tile * 16 + fe;
        float hv = 0.f;
        if (live) { hv = s_h[row * 16 + fe] + t0; s_h[row * 16 + fe] = hv; }
        float sq = hv * hv;
        sq += __shfl_xor(sq, 1, 64);
        sq += __shfl_xor(sq, 2, 64);
        sq += __shfl_xor(sq, 4, 64);
        sq += __shfl_xor(sq, 8, 64);
        if (more) {
          store_block(xgA_next, xgA_next + pl_d / 2, owner_tile, row, fe, hv * gn, live);
          if (live && fe == 0) st4f_coh(ssA_next + owner_tile * 32 + row, sq);
        } else if (live) {   // operand of the final norm, row-major, for the unembedding GEMM that follows
          bf16_t hi, lo;
          split_bf16(hv * gn, hi, lo);
          a.xg[(size_t)row * ld_a + n] = hi;
          a.xg[(size_t)row * ld_a + lo_a + n] = lo;
          if (fe == 0) a.ss[(size_t)row * NTd + owner_tile] = sq;
          a.h_out[(size_t)row * d + n] = hv;   // final residual rows, for inspection only
        }
      }
      if (more) prefetch_w(wpre, a.layers[l + 1].wqkv, KTd, min(wg, NT1 - 1));
    }
  }
}

#undef S2D2_ROLE

// Bytes of exchange buffers per layer: 2 operand planes x 2 (hi, lo), the SwiGLU output planes, the attention
// output, two blocked arrays of partial sums of squares.
size_t forward_fused_act_bytes(int d, int HqD, int F) {
  const size_t b = (size_t)4 * (d / 16) * 512 + (size_t)2 * (F / 16) * 512 + (size_t)16 * 2 * HqD * 2 + (size_t)2 * (d / 16) * 128;
  return (b + 255) & ~(size_t)255;
}

size_t forward_fused_lds() {
  const size_t merge = (size_t)FW * 2 * 256 * sizeof(float);
  return std::max(fa_lds(FW), merge);
}

__global__ void fused_set_layer_kernel(FusedLayer* dst, FusedLayer v) { *dst = v; }

void launch_fused_set_layer(hipStream_t st, FusedLayer* dst, const FusedLayer& v) {
  S2D2_LAUNCH(fused_set_layer_kernel, dim3(1), dim3(1), 0, st, dst, v);
}

int forward_fused_init() {
  return hipFuncSetAttribute((const void*)forward_fused_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)forward_fused_lds()) == hipSuccess ? 0 : -1;
}

// Workgroups of this kernel that fit one compute unit at a time (0 if the query fails).
int forward_fused_occupancy() {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, forward_fused_kernel, FW * 64, forward_fused_lds()) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return n;
}

void launch_forward_fused(hipStream_t st, const FusedArgs& a, int G) {
  S2D2_LAUNCH(forward_fused_kernel, dim3(G), dim3(FW * 64), forward_fused_lds(), st, a);
}

}  // namespace s2d2
