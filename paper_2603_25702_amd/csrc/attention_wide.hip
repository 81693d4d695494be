// Flash attention for windows with several 32-row query tiles (batched verification, large blocks).
//
// attn_flash_kernel gives every query tile a workgroup of its own, so a (sequence, KV head) pair with
// q_tiles query tiles reads its cached K / V q_tiles times.  Here the NW wavefronts of a workgroup each own
// ONE query tile of the same (sequence, KV head, key split) and walk the keys together: a 32-key tile of K
// and of V^T is fetched from global memory once per workgroup (every thread one or a few 16-byte pieces),
// parked in LDS, and read from there as MFMA operands by all wavefronts.  A wavefront never shares its
// softmax state, so there is no merge inside the workgroup; key splits merge through the same
// last-arriver scheme as the narrow kernel, in split order.
//
// Pipeline: two tiles are in flight in registers (sets R0 / R1) while a third is being consumed from one of two
// LDS buffers; a wavefront parks tile i + 1 in the other buffer after its own math on tile i, and one barrier
// per tile separates that from the reads of tile i + 1.  The page-table entries of the split's key range are copied to LDS
// once, so address generation never waits on a dependent global load.
#include "attention_flash.h"
#include <stdlib.h>
#include <type_traits>

namespace s2d2 {

#ifdef S2D2_KERNEL_TIMING
__device__ unsigned long long g_wide_ts[64];
// stamps of the first computing (k < 8) and the first fetching wavefront (k >= 8) of workgroup (0, 0, 0), tile 16
#define S2D2_WTS(k, cond) do { if ((cond) && lane == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) g_wide_ts[(k)] = wall_clock64(); } while (0)
__global__ void wide_ts_copy_kernel(unsigned long long* out) { if (threadIdx.x < 64) out[threadIdx.x] = g_wide_ts[threadIdx.x]; }
void launch_wide_ts_copy(hipStream_t st, void* out) { S2D2_LAUNCH(wide_ts_copy_kernel, dim3(1), dim3(64), 0, st, (unsigned long long*)out); }
#else
#define S2D2_WTS(k, cond) do {} while (0)
void launch_wide_ts_copy(hipStream_t, void*) {}
#endif

static constexpr int FW_KROW = 272;               // bytes per K row in LDS: 128 bf16 + 16 bytes (bank spread)
static constexpr int FW_VROW = 80;                // bytes per V^T row in LDS: 32 keys bf16 + 16 bytes
static constexpr int FW_KBUF = 32 * FW_KROW;
static constexpr int FW_BUF = FW_KBUF + 128 * FW_VROW;
static constexpr int FW_RING = 2;

size_t attention_wide_lds_bytes(int pt_cap) { return (size_t)FW_RING * FW_BUF + (size_t)pt_cap * 4 + 16; }

struct FwTile { bool win; int kbase, limit; };

// Keeps the first nv of 8 bf16 and zeroes the rest, without branches.
__device__ __forceinline__ uint4 fw_mask(uint4 v, int nv) {
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int k = nv - 2 * e;   // valid halves of this dword
    const uint32_t m = k >= 2 ? 0xffffffffu : (k == 1 ? 0xffffu : 0u);
    w[e] &= m;
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// 8 bf16 values (one 16-byte operand piece) as IEEE half: exact for magnitudes in the half range (the 8-bit
// significand fits), values below 2^-14 land on half subnormals (absolute error below 2^-24).
__device__ __forceinline__ uint32_t fw_bf16x2_to_f16x2(uint32_t w) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u)));
}
__device__ __forceinline__ uint4 fw_to_f16(uint4 v) {
  return make_uint4(fw_bf16x2_to_f16x2(v.x), fw_bf16x2_to_f16x2(v.y), fw_bf16x2_to_f16x2(v.z), fw_bf16x2_to_f16x2(v.w));
}

// QM: how the queries come and the arithmetic type of both products.  OPM_BF16 / OPM_BF16X2: bf16 MFMA on the
// cache's bf16 keys and values, queries and softmax weights as one or as a high + low bf16 plane.  OPM_F16: queries
// as IEEE half, keys and values converted to half on their way into LDS (by the fetching wavefronts), softmax
// weights as half: one 11-bit plane on the f16 MFMA, half the matrix instructions of the two-plane form and no
// high / low split of the weights.
template <int NW, int QM>
__global__ __launch_bounds__(NW * 64, 2) void attn_flash_wide_kernel(
    const bf16_t* __restrict__ q, int q_ld, int q_lo, const bf16_t* __restrict__ k_win, const bf16_t* __restrict__ vT_win,
    const bf16_t* __restrict__ k_pages, const bf16_t* __restrict__ v_pages, KvGeom g, Plan p, int Hq, int Z,
    int wpad, float scale_log2e, bf16_t* __restrict__ o, int o_ld, int o_lo, float* __restrict__ part_o,
    float* __restrict__ part_ml, int32_t* __restrict__ counters, int q_tiles, int per, int pt_cap, int ps_shift) {
  constexpr int D = FA_D, T = NW * 64, U = 512 / T;
  constexpr bool SPLIT = QM == OPM_BF16X2, F16 = QM == OPM_F16;
  static_assert(U == 1 || U == 2, "8 or 4 wavefronts");
  extern __shared__ __align__(16) unsigned char lds[];
  int32_t* s_pt = (int32_t*)(lds + FW_RING * FW_BUF);
  int* s_last = (int*)(s_pt + pt_cap);
  const int z = blockIdx.x, qgrp = blockIdx.y, item = blockIdx.z;
  const int Hkv = g.n_kv_heads, ps = g.page_size;
  const int n = item / Hkv, kvh = item % Hkv;
  const int grp = Hq / Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, h = lane >> 5;
  const int cap = g.max_pages_per_seq * ps;
  const int S = max(0, min(g.seq_len[n], cap));
  const int row0 = p.seq_row0[n], nw = p.seq_rows[n];
  const int nq = nw * grp;
  // query tiles qgrp * per .. + per of this (sequence, KV head) belong to this workgroup, one per wavefront (per <= NW)
  if (qgrp * per * 32 >= nq) return;            // the whole workgroup: nothing to do (before any barrier)
  const int qt = qgrp * per + wave, q0 = qt * 32;
  const bool active = wave < per && q0 < nq;
  const int qi = min(q0 + c, nq - 1);
  const int r = row0 + qi / grp, head = kvh * grp + qi % grp;
  const int lo = p.row_lo[r], hi = p.row_hi[r];

  const int Tc = (S + 31) >> 5, Tw = (nw + 31) >> 5;
  const int t0 = (int)((long long)Tc * z / Z), t1 = (int)((long long)Tc * (z + 1) / Z);
  const int n_c = t1 - t0, n_w = z == Z - 1 ? Tw : 0, n_it = n_c + n_w;

  // page-table slice of this split's keys
  const int pb0 = (t0 * 32) >> ps_shift;   // page_size = 1 << ps_shift
  {
    const int pe = (min(t1 * 32, cap) + ps - 1) >> ps_shift;
    const int32_t* pt = g.page_table + (size_t)n * g.max_pages_per_seq;
    for (int i = tid; i < min(pe - pb0, pt_cap); i += T) s_pt[i] = min(max(pt[pb0 + i], 0), g.n_pages - 1);
  }

  uint4 qf[8], ql[SPLIT ? 8 : 1];
  {
    const bf16_t* qp = q + (size_t)r * q_ld + head * D + 8 * h;
#pragma unroll
    for (int ds = 0; ds < 8; ++ds) {
      qf[ds] = *(const uint4*)(qp + ds * 16);
      if (SPLIT) ql[ds] = *(const uint4*)(qp + q_lo + ds * 16);
    }
  }
  FaState st;
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o[t][i] = 0.f;
  __syncthreads();   // s_pt

  // (closures capture scalars by value: captured references would pin the locals to memory)
  // Leading tiles of this split that are full tiles of cached keys (all but, at most, the last cached tile of the
  // last split).  The loops below run them through forms of fetch / park / compute that are compiled for exactly
  // that case (FAST): no clamps, no second address form, no visibility mask.  Both kinds of wavefronts are bound
  // by their vector-ALU instructions, not by the matrix pipes or by memory.
  const int n_fast = max(0, min(n_c, (S >> 5) - t0));
  auto tile_fast = [=](int i) __attribute__((always_inline)) {
    FwTile t;
    t.win = false;
    t.kbase = (t0 + i) * 32;
    t.limit = S;
    return t;
  };
  auto tile_of = [=](int i) __attribute__((always_inline)) {
    FwTile t;
    i = min(i, n_it - 1);
    t.win = i >= n_c;
    t.kbase = (t.win ? i - n_c : t0 + i) * 32;
    t.limit = t.win ? nw : S;
    return t;
  };
  // piece idx of a tile: K row idx / 16, 16-byte piece idx % 16;  V^T row idx / 4, keys 8 (idx % 4) .. + 8.
  // Thread tid handles pieces tid + u T, u < U (each piece in a named register set, never an indexed array).
  // (offsets are written as  page * page_stride + [terms that depend on the thread alone] + [32-bit terms of the
  // tile]: the middle part is computed once per thread ahead of the loop, and a piece costs one table look-up and
  // one 64-bit multiply-add per tile; the fetching wavefronts share their SIMDs with the computing ones)
  const size_t pstride = (size_t)Hkv * ps * D;   // elements of a page
  auto fetchp = [=](auto fast, int idx, int i, uint4& kr, uint4& vr) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast)::value;
    const int kk = idx >> 4, kch = idx & 15, vd = idx >> 2, vko = (idx & 3) * 8;
    if (FAST) {
      const int key = (t0 + i) * 32 + kk, kv0 = (t0 + i) * 32 + vko;
      const int pk = s_pt[min((key >> ps_shift) - pb0, pt_cap - 1)];
      const int pv = s_pt[min((kv0 >> ps_shift) - pb0, pt_cap - 1)];
      kr = *(const uint4*)(k_pages + ((size_t)kvh * ps * D + kch * 8) + (size_t)pk * pstride + (key & (ps - 1)) * D);
      vr = *(const uint4*)(v_pages + ((size_t)kvh * D + vd) * ps + (size_t)pv * pstride + (kv0 & (ps - 1)));
      return;
    }
    const FwTile t = tile_of(i);
    const int key = min(t.kbase + kk, t.limit - 1);   // rows beyond the region read a valid row; their scores are masked
    const int key0 = t.kbase + vko;
    // both address forms are computed and one is selected: no control flow around the loads
    const int kv0 = min(key0, cap - 8);
    const int pk = s_pt[max(0, min((key >> ps_shift) - pb0, pt_cap - 1))];
    const int pv = s_pt[max(0, min((kv0 >> ps_shift) - pb0, pt_cap - 1))];
    const bf16_t* kp_c = k_pages + ((size_t)kvh * ps * D + kch * 8) + (size_t)pk * pstride + (key & (ps - 1)) * D;
    const bf16_t* vp_c = v_pages + ((size_t)kvh * D + vd) * ps + (size_t)pv * pstride + (kv0 & (ps - 1));
    const bf16_t* kp_w = k_win + ((size_t)row0 * Hkv + kvh) * D + kch * 8 + (size_t)key * (Hkv * D);
    const bf16_t* vp_w = vT_win + ((size_t)(n * Hkv + kvh) * D + vd) * wpad + min(key0, wpad - 8);
    kr = *(const uint4*)(t.win ? kp_w : kp_c);
    vr = *(const uint4*)(t.win ? vp_w : vp_c);
  };
  auto fetch1 = [=](auto fast, int u, int i, uint4& kr, uint4& vr) __attribute__((always_inline)) { fetchp(fast, min(tid + u * T, 511), i, kr, vr); };
  auto stashp = [=](auto fast, int idx, int i, int b, uint4 kr, uint4 vr) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast)::value;
    unsigned char* base = lds + b * FW_BUF;
    const int kk = idx >> 4, kch = idx & 15, vd = idx >> 2, vko = (idx & 3) * 8;
    if (FAST) {
      *(uint4*)(base + kk * FW_KROW + kch * 16) = F16 ? fw_to_f16(kr) : kr;
      *(uint4*)(base + FW_KBUF + vd * FW_VROW + vko * 2) = F16 ? fw_to_f16(vr) : vr;
      return;
    }
    const FwTile t = tile_of(i);
    // half mode: cached tiles are bf16 and are converted here; the window's own rows already come as half values
    // (k_win / vT_win then point at the half copies the QKV projection wrote: 11 bits instead of the cache's 8)
    const uint4 vm = t.kbase + 32 <= t.limit ? vr : fw_mask(vr, t.limit - (t.kbase + vko));   // (uniform: only a region's last tile is partial)
    const bool cvt = F16 && !t.win;
    *(uint4*)(base + kk * FW_KROW + kch * 16) = cvt ? fw_to_f16(kr) : kr;
    *(uint4*)(base + FW_KBUF + vd * FW_VROW + vko * 2) = cvt ? fw_to_f16(vm) : vm;
  };
  auto stash1 = [=](auto fast, int u, int i, int b, uint4 kr, uint4 vr) __attribute__((always_inline)) { stashp(fast, min(tid + u * T, 511), i, b, kr, vr); };   // clamped duplicates rewrite the same bytes
  const int kperm = fa_perm(c);
  auto compute = [=](auto fast, FaState& st, const uint4 (&qf)[8], const uint4 (&ql)[SPLIT ? 8 : 1], int i, int b) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast)::value;
    const FwTile t = FAST ? tile_fast(i) : tile_of(i);
    const unsigned char* kb = lds + b * FW_BUF + kperm * FW_KROW + 16 * h;
    const unsigned char* vb = lds + b * FW_BUF + FW_KBUF + c * FW_VROW + 16 * h;
    f32x16_t sacc;
    S2D2_WTS(0, FAST && wave == 0 && i == 16);
#pragma unroll
    for (int j = 0; j < 16; ++j) sacc[j] = 0.f;
#pragma unroll
    for (int ds = 0; ds < 8; ++ds) {
      const uint4 kraw = *(const uint4*)(kb + ds * 32);
      if (F16) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, kraw), __builtin_bit_cast(f16x8_t, qf[ds]), sacc, 0, 0, 0);
      } else {
        const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, kraw);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, __builtin_bit_cast(bf16x8_t, qf[ds]), sacc, 0, 0, 0);
        if (SPLIT) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, __builtin_bit_cast(bf16x8_t, ql[ds]), sacc, 0, 0, 0);
      }
    }
    // sacc[j]: key kbase + 16 (j / 8) + 8 h + (j % 8), query row c.  Scores stay unscaled until the exponent:
    // the running maximum is kept in scaled units, exp2(s * scale - m) is one fused multiply-add per element.
#ifdef S2D2_KERNEL_TIMING
    if (sacc[0] == 12345.678f) return;
    S2D2_WTS(1, FAST && wave == 0 && i == 16);
#endif
    float mx = -INFINITY;
    if (FAST || (!t.win && t.kbase + 32 <= t.limit)) {   // a full tile of cached keys: every key is visible
#pragma unroll
      for (int j = 0; j < 16; ++j) mx = fmaxf(mx, sacc[j]);
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int key = t.kbase + 16 * (j >> 3) + 8 * h + (j & 7);
        const int w = row0 + key;
        const int vis = (int)!t.win | ((int)(w >= lo) & (int)(w < hi)) | (int)(w == r);
        sacc[j] = ((int)(key < t.limit) & vis) ? sacc[j] : -INFINITY;
        mx = fmaxf(mx, sacc[j]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2e;
    // no divergent control flow around the MFMAs: a query row that sees nothing yet keeps m = -inf
    // and uses 0 as the reference, which makes every p below exp2(-inf) = 0
    const float m_new = fmaxf(st.m, mx);
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_ref);
    float ls = 0.f;
    bf16x8_t pb[2], pl[SPLIT ? 2 : 1];
    f16x8_t ph16[2];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[j], scale_log2e, -m_ref));
      ls += pv;
      if (F16) {
        ph16[j >> 3][j & 7] = (_Float16)pv;
      } else {
        const __bf16 ph = (__bf16)pv;
        pb[j >> 3][j & 7] = ph;
        if (SPLIT) pl[j >> 3][j & 7] = (__bf16)(pv - (float)ph);
      }
    }
    ls += __shfl_xor(ls, 32, 64);
    st.l = st.l * alpha + ls;
    st.m = m_new;
#ifdef S2D2_KERNEL_TIMING
    if (ls == 12345.678f) return;
    S2D2_WTS(2, FAST && wave == 0 && i == 16);
#endif
    // the accumulators are rescaled only when some row's maximum moved (alpha = 1 leaves them as they are)
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int j = 0; j < 16; ++j) st.o[dt][j] *= alpha;
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const uint4 vraw = *(const uint4*)(vb + dt * 32 * FW_VROW + j * 32);
        if (F16) {
          st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, vraw), ph16[j], st.o[dt], 0, 0, 0);
        } else {
          const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, vraw);
          st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[j], st.o[dt], 0, 0, 0);
          if (SPLIT) st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pl[j], st.o[dt], 0, 0, 0);
        }
      }
    }
#ifdef S2D2_KERNEL_TIMING
    if (st.o[3][15] == 12345.678f) return;
    S2D2_WTS(3, FAST && wave == 0 && i == 16);
#endif
  };

  // A workgroup of 8 wavefronts of which at most half own a query tile with rows (a fresh block fills 4 of the
  // verifier's 6 tiles): the upper half of the wavefronts does all the fetching, PP pieces per thread in two
  // register sets, and the wavefronts that compute do nothing else.  With every wavefront fetching its share, the
  // address arithmetic and LDS stores of the fetch sat on the critical wavefronts; workgroups without idle
  // wavefronts were slower still for the same reason.  (The same split in 4-wavefront workgroups, two fetching
  // wavefronts with four pieces each, measured slower on two of three configurations and is not used.)
  const int n_live = min(per, (nq - qgrp * per * 32 + 31) >> 5);
  const bool spec = NW == 8 && 2 * n_live <= NW;
  constexpr std::true_type FT_{};
  constexpr std::false_type GT_{};
  if (n_it > 0 && spec) {
    if (wave >= NW / 2) {
      constexpr int PP = 16 / NW;                       // pieces per fetching thread
      const int pbase = tid - NW * 32;                  // 0 .. NW*32 - 1; piece u of this thread: pbase + u * NW * 32
      uint4 ak[PP], av[PP], bk[PP], bv[PP];             // (indices are compile-time constants throughout)
#pragma unroll
      for (int u = 0; u < PP; ++u) fetchp(GT_, pbase + u * NW * 32, 0, ak[u], av[u]);
#pragma unroll
      for (int u = 0; u < PP; ++u) fetchp(GT_, pbase + u * NW * 32, 1, bk[u], bv[u]);
#pragma unroll
      for (int u = 0; u < PP; ++u) stashp(GT_, pbase + u * NW * 32, 0, 0, ak[u], av[u]);
#pragma unroll
      for (int u = 0; u < PP; ++u) fetchp(GT_, pbase + u * NW * 32, 2, ak[u], av[u]);
      __syncthreads();
      // one pass: parks tiles i + 1, i + 2 and requests tiles i + 3, i + 4
      auto pass = [&](auto fast, int i) __attribute__((always_inline)) {
        S2D2_WTS(8, wave == NW / 2 && i == 16);
#pragma unroll
        for (int u = 0; u < PP; ++u) stashp(fast, pbase + u * NW * 32, i + 1, 1, bk[u], bv[u]);
        S2D2_WTS(9, wave == NW / 2 && i == 16);
#pragma unroll
        for (int u = 0; u < PP; ++u) fetchp(fast, pbase + u * NW * 32, i + 3, bk[u], bv[u]);
        S2D2_WTS(10, wave == NW / 2 && i == 16);
        __syncthreads();
        S2D2_WTS(11, wave == NW / 2 && i == 16);
        if (i + 1 < n_it) {
#pragma unroll
          for (int u = 0; u < PP; ++u) stashp(fast, pbase + u * NW * 32, i + 2, 0, ak[u], av[u]);
#pragma unroll
          for (int u = 0; u < PP; ++u) fetchp(fast, pbase + u * NW * 32, i + 4, ak[u], av[u]);
          S2D2_WTS(12, wave == NW / 2 && i == 16);
          __syncthreads();
          S2D2_WTS(13, wave == NW / 2 && i == 16);
        }
      };
      int i = 0;
      for (; i + 4 < n_fast; i += 2) pass(FT_, i);
      for (; i < n_it; i += 2) pass(GT_, i);
    } else {
      __syncthreads();
      auto pass = [&](auto fast, int i) __attribute__((always_inline)) {
        if (active) compute(fast, st, qf, ql, i, 0);
        __syncthreads();
        S2D2_WTS(4, wave == 0 && i == 16);
        if (i + 1 < n_it) {
          if (active) compute(fast, st, qf, ql, i + 1, 1);
          __syncthreads();
          S2D2_WTS(5, wave == 0 && i == 16);
        }
      };
      int i = 0;
      for (; i + 4 < n_fast; i += 2) pass(FT_, i);   // (the same split of the passes as in the fetching wavefronts: equal barrier counts)
      for (; i < n_it; i += 2) pass(GT_, i);
    }
  } else if (n_it > 0) {
    if constexpr (U == 1) {
      // two tiles in flight in registers: set B holds tile i + 1 and set A tile i + 2 at the top of an (even) iteration
      uint4 ak, av, bk, bv;
      fetch1(GT_, 0, 0, ak, av);
      fetch1(GT_, 0, 1, bk, bv);
      stash1(GT_, 0, 0, 0, ak, av);
      fetch1(GT_, 0, 2, ak, av);
      __syncthreads();
      auto pass = [&](auto fast, int i) __attribute__((always_inline)) {
        if (active) compute(fast, st, qf, ql, i, 0);
        stash1(fast, 0, i + 1, 1, bk, bv);
        fetch1(fast, 0, i + 3, bk, bv);
        __syncthreads();
        if (i + 1 < n_it) {
          if (active) compute(fast, st, qf, ql, i + 1, 1);
          stash1(fast, 0, i + 2, 0, ak, av);
          fetch1(fast, 0, i + 4, ak, av);
          __syncthreads();
        }
      };
      int i = 0;
      for (; i + 4 < n_fast; i += 2) pass(FT_, i);
      for (; i < n_it; i += 2) pass(GT_, i);
    } else {
      // smaller workgroups hold several pieces per thread: one tile in flight (two workgroups share a CU)
      uint4 k0, v0, k1, v1;
      fetch1(GT_, 0, 0, k0, v0);
      fetch1(GT_, 1, 0, k1, v1);
      stash1(GT_, 0, 0, 0, k0, v0);
      stash1(GT_, 1, 0, 0, k1, v1);
      fetch1(GT_, 0, 1, k0, v0);
      fetch1(GT_, 1, 1, k1, v1);
      __syncthreads();
      // one pass: computes tile i, parks tile i + 1, requests tile i + 2
      auto pass = [&](auto fast, int i) __attribute__((always_inline)) {
        if (active) compute(fast, st, qf, ql, i, i & 1);
        stash1(fast, 0, i + 1, (i + 1) & 1, k0, v0);
        stash1(fast, 1, i + 1, (i + 1) & 1, k1, v1);
        fetch1(fast, 0, i + 2, k0, v0);
        fetch1(fast, 1, i + 2, k1, v1);
        __syncthreads();
      };
      int i = 0;
      for (; i + 2 < n_fast; ++i) pass(FT_, i);
      for (; i < n_it; ++i) pass(GT_, i);
    }
  }

  // ---- output: lane (c, h) holds head-dim positions dt*32 + 8*i4 + 4*h .. + 4 of query row c ----
  const size_t item0 = ((size_t)item * q_tiles + qt) * Z;
  if (Z == 1) {
    if (active && q0 + c < nq) {
      const float inv = st.l > 0.f ? 1.0f / st.l : 0.f;
      bf16_t* op = o + (size_t)r * o_ld + head * D + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          fa_store4<false>(op + dt * 32 + 8 * i4, o_lo, st.o[dt][4 * i4] * inv, st.o[dt][4 * i4 + 1] * inv,
                           st.o[dt][4 * i4 + 2] * inv, st.o[dt][4 * i4 + 3] * inv);
    }
    return;
  }
  if (active) {
    float* po = part_o + (item0 + z) * 32 * D + (size_t)lane * 4;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        st16f_coh(po + (dt * 4 + i4) * 256, st.o[dt][4 * i4], st.o[dt][4 * i4 + 1], st.o[dt][4 * i4 + 2], st.o[dt][4 * i4 + 3]);
    if (h == 0) {
      st4f_coh(&part_ml[(item0 + z) * 64 + c], st.m);
      st4f_coh(&part_ml[(item0 + z) * 64 + 32 + c], st.l);
    }
  }
  __builtin_amdgcn_s_waitcnt(0);  // the write-through stores of the partials have completed before the arrival is counted
  __syncthreads();
  const int cidx = item * q_tiles + qgrp * per;
  if (tid == 0) {
    const int prev = __hip_atomic_fetch_add(&counters[cidx], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_last = prev == Z - 1;
    if (prev == Z - 1) __hip_atomic_store(&counters[cidx], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (!*s_last) return;
  // the last split to arrive merges every query tile of the workgroup, all threads on one tile at a time
  for (int w = 0; w < per; ++w) {
    const int qt2 = qgrp * per + w;
    if (qt2 * 32 >= nq) break;
    // in passes of 512 pieces, so that a thread never holds more than two pieces per split in registers
#pragma unroll 1
    for (int pass = 0; pass < 512 / T; ++pass)
      fa_combine<false, 512>(part_o, part_ml, ((size_t)item * q_tiles + qt2) * Z, Z, tid + pass * T, qt2, nq, grp, row0, kvh, Hq, o, o_ld, o_lo);
  }
}

template <int NW>
static void launch_wide(hipStream_t st, int qm, dim3 grid, size_t lds, const bf16_t* q, int q_ld, int q_lo,
                        const bf16_t* k_win, const bf16_t* vT_win, const bf16_t* kp, const bf16_t* vp, const KvGeom& g,
                        const Plan& p, int Hq, int Z, int wpad, float scale_log2e, bf16_t* o, int o_ld, int o_lo,
                        float* part_o, float* part_ml, int32_t* counters, int q_tiles, int per, int pt_cap, int ps_shift) {
#define S2D2_WIDE_QM(QMV)                                                                                                    \
  S2D2_LAUNCH((attn_flash_wide_kernel<NW, QMV>), grid, dim3(NW * 64), lds, st, q, q_ld, q_lo, k_win, vT_win, kp, vp, g, p, \
              Hq, Z, wpad, scale_log2e, o, o_ld, o_lo, part_o, part_ml, counters, q_tiles, per, pt_cap, ps_shift)
  if (qm == OPM_F16) S2D2_WIDE_QM(OPM_F16);
  else if (qm == OPM_BF16X2) S2D2_WIDE_QM(OPM_BF16X2);
  else S2D2_WIDE_QM(OPM_BF16);
#undef S2D2_WIDE_QM
}

// Wavefronts per workgroup for q_tiles query tiles: as few query groups as 8-wavefront workgroups allow,
// then the smallest supported workgroup that covers a group.
int attention_wide_nw(int q_tiles) {
  const int groups = (q_tiles + 7) / 8, need = (q_tiles + groups - 1) / groups;
  return need <= 4 ? 4 : 8;   // (two wavefronts for two tiles measured slower: four share the fetch work, 3.76 -> 3.27 ms of attention per step on the 4B shape)
}

// Page-table entries a split can touch (plus slack for the ragged ends).
int attention_wide_pt_cap(const KvGeom& g, int Z) {
  const int cap_tiles = (g.max_pages_per_seq * g.page_size + 31) / 32;
  const int per_split = (cap_tiles + Z - 1) / Z + 1;
  return std::min(g.max_pages_per_seq, per_split * 32 / g.page_size + 2);
}

void launch_attention_wide(hipStream_t st, const void* q, int q_ld, int q_lo, const void* k_win, const void* vT_win,
                           const void* k_pages_layer, const void* v_pages_layer, const KvGeom& g, const Plan& p, int N,
                           int Hq, int q_tiles, int Z, int wpad, void* o, int o_ld, int o_lo, float* part,
                           size_t part_entries, int32_t* counters) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)g.head_dim);
  const int items = N * g.n_kv_heads;
  const int qgroups = (q_tiles + 7) / 8, per = (q_tiles + qgroups - 1) / qgroups;   // tiles per workgroup, balanced
  const int nw = attention_wide_nw(q_tiles);
  const int pt_cap = attention_wide_pt_cap(g, Z);
  float* part_o = part;
  float* part_ml = part + part_entries * 32 * FA_D;
  const dim3 grid(Z, qgroups, items);
  const size_t lds = attention_wide_lds_bytes(pt_cap);
  int ps_shift = 0;
  while ((1 << ps_shift) < g.page_size) ++ps_shift;   // the caller has checked that page_size is a power of two
#define S2D2_WIDE(NWV)                                                                                                  \
  launch_wide<NWV>(st, operand_mode(q_lo), grid, lds, (const bf16_t*)q, q_ld, q_lo, (const bf16_t*)k_win, (const bf16_t*)vT_win, \
                   (const bf16_t*)k_pages_layer, (const bf16_t*)v_pages_layer, g, p, Hq, Z, wpad, scale_log2e,          \
                   (bf16_t*)o, o_ld, o_lo, part_o, part_ml, counters, q_tiles, per, pt_cap, ps_shift)
  if (nw == 4) S2D2_WIDE(4);
  else S2D2_WIDE(8);
#undef S2D2_WIDE
}

template <int NW, int QM>
static hipError_t wide_lds_limit() {
  return hipFuncSetAttribute((const void*)attn_flash_wide_kernel<NW, QM>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

int attention_wide_init() {
  hipError_t e = hipSuccess;
#define S2D2_LIM(NWV)                                                          \
  if (e == hipSuccess) e = wide_lds_limit<NWV, OPM_BF16>();                    \
  if (e == hipSuccess) e = wide_lds_limit<NWV, OPM_BF16X2>();                  \
  if (e == hipSuccess) e = wide_lds_limit<NWV, OPM_F16>();
  S2D2_LIM(4) S2D2_LIM(8)
#undef S2D2_LIM
  return e == hipSuccess ? 0 : -1;
}

}  // namespace s2d2
