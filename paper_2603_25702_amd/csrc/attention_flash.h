// MFMA flash attention over the paged prefix cache plus the window: device-side body of the kernel in attention.hip.
#pragma once
#include "s2d2_internal.h"

namespace s2d2 {

#ifdef S2D2_KERNEL_TIMING
__device__ unsigned long long g_attn_ts[64];
#define S2D2_ATS(k) do { if (threadIdx.x == 0 && z == 0 && item_zy == 0) g_attn_ts[k] = wall_clock64(); } while (0)
#define S2D2_ATS_ANY(k) do { if (threadIdx.x == 0 && item_zy == 0) g_attn_ts[k] = wall_clock64(); } while (0)
#else
#define S2D2_ATS(k) do {} while (0)
#define S2D2_ATS_ANY(k) do {} while (0)
#endif

// ---------------------------------------------------------------------------------------------
// attn_flash_kernel (bf16, head_dim 128): split-key flash attention on 32x32x16 MFMA.
//
// Work item = (sequence, KV head, tile of 32 query rows, key split).  A "query row" is a
// (window row, query head of the group) pair, so GQA groups share every K/V byte.  Each of the
// NW wavefronts of a workgroup takes every NW-th tile of 32 keys of its split, streams K and V
// straight from global memory into MFMA operands (no LDS on the K/V path), and keeps an online
// softmax state.  Scores are computed transposed, S^T = K Q^T, so that one lane owns one query
// row: its running max / sum and the rescaling of its output column need no cross-lane traffic
// beyond one exchange between the two half-waves.  The rows of the K tile are fed in a permuted
// order chosen so that the fp32 S^T accumulators of a lane, packed to bf16, are exactly the B
// operand (8 consecutive keys) of O^T = V^T P^T; the cache stores V key-minor ([D, page_size])
// so that the matching A operand is one 16-byte load.  Wavefronts merge through LDS in wavefront
// order; key splits are merged, in split order, by the workgroup of a tile that arrives last at the tile's counter.
// ---------------------------------------------------------------------------------------------
static constexpr int FA_D = 128;

__device__ __forceinline__ int fa_perm(int rr) {  // MFMA row -> key offset inside the 32-key tile
  const int a = rr >> 3, hh = (rr >> 2) & 1, b = rr & 3;
  return (a >> 1) * 16 + hh * 8 + (a & 1) * 4 + b;
}

__device__ __forceinline__ uint4 mask_keys(uint4 v, int nv) {  // keep the first nv of 8 bf16, zero the rest
  if (nv >= 8) return v;
  if (nv <= 0) return make_uint4(0, 0, 0, 0);
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int k = nv - 2 * e;  // valid halves in this dword
    w[e] = k >= 2 ? w[e] : (k == 1 ? (w[e] & 0xffffu) : 0u);
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// x / d for 0 <= x < 2^20 and d >= 1, exact, without the long reciprocal sequence of an integer division (the
// divisor below is only known once seq_len has arrived, so nothing of that sequence could be hoisted above the wait).
__device__ __forceinline__ int fa_div(int x, int d) {
  int q = (int)((float)x * __builtin_amdgcn_rcpf((float)d));
  q -= (int)(q * d > x);
  q += (int)((q + 1) * d <= x);
  return q;
}

struct FaState {
  float m, l;
  f32x16_t o[4];
};

__device__ __forceinline__ void fa_merge(FaState& a, float m2, float l2, const f32x16_t* o2) {
  const float M = fmaxf(a.m, m2);
  const float f1 = a.m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(a.m - M);
  const float f2 = m2 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - M);
  a.l = a.l * f1 + l2 * f2;
  a.m = M;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) a.o[t][i] = a.o[t][i] * f1 + o2[t][i] * f2;
}

// Four consecutive output elements in the storage the low-plane offset o_lo names (bf16, bf16 hi + lo planes, or half).
template <bool COH>
__device__ __forceinline__ void fa_store4(bf16_t* p, int o_lo, float a, float b, float c, float d) {
  uint2 first, second;
  act_pack4(o_lo, a, b, c, d, first, second);
  if (COH) st8_coh(p, first); else *(uint2*)p = first;
  if (o_lo > 0) {
    if (COH) st8_coh(p + o_lo, second); else *(uint2*)(p + o_lo) = second;
  }
}

// Merges the Z split partials of one (sequence, KV head, query tile) in split order.  All loads of a thread's
// items are issued before any of them is used (one memory round trip for up to ZMAX splits); more splits
// take further rounds of ZMAX.
template <bool COH, int NTHREADS>
__device__ __forceinline__ void fa_combine(const float* part_o, const float* part_ml, size_t item0, int Z, int tid,
                                           int qt, int nq, int grp, int row0, int kvh, int Hq,
                                           bf16_t* __restrict__ o, int o_ld, int o_lo) {
  constexpr int D = FA_D, ITEMS = 32 * (D / 4) / NTHREADS, ZMAX = 4;
  static_assert(ITEMS >= 1 && ITEMS * NTHREADS == 32 * (D / 4), "thread count must divide the 1024 output chunks");
  float M[ITEMS], l[ITEMS];
  float4 acc[ITEMS];
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) { M[it] = -INFINITY; l[it] = 0.f; acc[it] = make_float4(0.f, 0.f, 0.f, 0.f); }
  for (int z0 = 0; z0 < Z; z0 += ZMAX) {
    float m[ITEMS][ZMAX], lz[ITEMS][ZMAX];
    uint4 pq[ITEMS][ZMAX];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int e = tid + it * NTHREADS, c = e & 31;   // element e: lane e % 64 = 32 h + c, group e / 64 = dt*4 + i4
#pragma unroll
      for (int k = 0; k < ZMAX; ++k) {
        const int z = min(z0 + k, Z - 1);   // clamped duplicates are skipped below
        m[it][k] = ld4f_coh(&part_ml[(item0 + z) * 64 + c]);
        lz[it][k] = ld4f_coh(&part_ml[(item0 + z) * 64 + 32 + c]);
        pq[it][k] = ld16_coh(part_o + (item0 + z) * 32 * D + (size_t)e * 4);
      }
    }
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
#pragma unroll
      for (int k = 0; k < ZMAX; ++k) {   // in split order: running rescale
        if (z0 + k >= Z || m[it][k] == -INFINITY) continue;
        const float Mn = fmaxf(M[it], m[it][k]);
        const float fo = M[it] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(M[it] - Mn);
        const float fn = __builtin_amdgcn_exp2f(m[it][k] - Mn);
        l[it] = l[it] * fo + fn * lz[it][k];
        acc[it].x = acc[it].x * fo + fn * __uint_as_float(pq[it][k].x);
        acc[it].y = acc[it].y * fo + fn * __uint_as_float(pq[it][k].y);
        acc[it].z = acc[it].z * fo + fn * __uint_as_float(pq[it][k].z);
        acc[it].w = acc[it].w * fo + fn * __uint_as_float(pq[it][k].w);
        M[it] = Mn;
      }
    }
  }
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int e = tid + it * NTHREADS, c = e & 31, g16 = e >> 6;
    const int d0 = (g16 >> 2) * 32 + 8 * (g16 & 3) + 4 * ((e >> 5) & 1);
    const int qi = qt * 32 + c;
    if (qi >= nq) continue;
    const float inv = l[it] > 0.f ? 1.0f / l[it] : 0.f;
    const int r = row0 + qi / grp, head = kvh * grp + qi % grp;
    fa_store4<COH>(o + (size_t)r * o_ld + head * D + d0, o_lo, acc[it].x * inv, acc[it].y * inv, acc[it].z * inv, acc[it].w * inv);
  }
}

// SPLIT: queries and softmax weights are used as high + low bf16 planes (16 significant bits): the
// score and the P*V products are each issued twice against the same K / V operands.
// COH: q, the window K / V and o are read and written with device-coherent accesses (for a caller whose producer
// or consumer is another workgroup of the SAME launch; the stand-alone kernel passes false).  The split partials
// always are.
// (z, qt, item) = (key split, query tile, sequence * Hkv + KV head); q_tiles = query tiles per item.
template <int NW, bool SPLIT, bool COH>
__device__ __forceinline__ void attn_flash_body(
    const bf16_t* __restrict__ q, int q_ld, int q_lo, const bf16_t* __restrict__ k_win, const bf16_t* __restrict__ vT_win,
    const bf16_t* __restrict__ k_pages, const bf16_t* __restrict__ v_pages, const KvGeom& g, const Plan& p, int Hq, int Z,
    int wpad, float scale_log2e, bf16_t* __restrict__ o, int o_ld, int o_lo, float* __restrict__ part_o,
    float* __restrict__ part_ml, int32_t* __restrict__ counters, int z, int qt, int item_zy, int q_tiles, float* smem) {
  constexpr int D = FA_D;
  S2D2_ATS(0);
  const int Hkv = g.n_kv_heads, ps = g.page_size;
  const int n = item_zy / Hkv, kvh = item_zy % Hkv;
  const int grp = Hq / Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 31, h = lane >> 5;
  const int32_t* pt = g.page_table + (size_t)n * g.max_pages_per_seq;
  // Tile t of the cached keys belongs to wavefront (t mod GW) of the GW = Zeff * NW wavefronts (Zeff <= Z, below) that
  // share this (sequence, KV head, query tile): the assignment does not depend on seq_len, so the
  // page-table entries of a wavefront's first tile are requested together with seq_len and the
  // plan entries (one round trip), and K / V follow in the second.
  const int gw = z * NW + wave;
  const int kperm = fa_perm(c);
  const int cap = g.max_pages_per_seq * ps;
  int page_k = pt[min(gw * 32 + kperm, cap - 1) / ps];
  int page_v[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) page_v[j] = pt[min(gw * 32 + 16 * j + 8 * h, cap - 1) / ps];
  const int S = max(0, min(g.seq_len[n], cap));
  const int row0 = p.seq_row0[n], nw = p.seq_rows[n];
  const int nq = nw * grp, q0 = qt * 32;
  if (q0 >= nq) return;
  const int qi = min(q0 + c, nq - 1);
  const int r = row0 + qi / grp, head = kvh * grp + qi % grp;
  const int lo = p.row_lo[r], hi = p.row_hi[r];

  uint4 qf[8], ql[SPLIT ? 8 : 1];
  {
    const bf16_t* qp = q + (size_t)r * q_ld + head * D + 8 * h;
#pragma unroll
    for (int ds = 0; ds < 8; ++ds) {
      qf[ds] = COH ? ld16_coh(qp + ds * 16) : *(const uint4*)(qp + ds * 16);
      if (SPLIT) ql[ds] = COH ? ld16_coh(qp + q_lo + ds * 16) : *(const uint4*)(qp + q_lo + ds * 16);
    }
  }
  if (qf[0].x == 0x12345678u && S < 0) return;   // (timing aid: forces the header and q loads to complete)
  S2D2_ATS(1);
  FaState st;
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o[t][i] = 0.f;

  const int Tc = (S + 31) >> 5, Tw = (nw + 31) >> 5;
  // The host sizes Z for the cache's CAPACITY; a sequence far below it uses only the first Zeff splits, the others
  // leave at once and are neither waited for nor merged.  Up to four splits (one round of the merge below) as soon as
  // every second wavefront has a tile, more only when a wavefront would otherwise walk several tiles.
  const int T_all = Tc + Tw;
  const int Zeff = max(1, min(Z, max((T_all + NW - 1) / NW, min(4, (2 * T_all + NW - 1) / NW))));
  if (z >= Zeff) return;
  const int GW = Zeff * NW;
  const int n_c = Tc > gw ? fa_div(Tc - gw + GW - 1, GW) : 0;      // cached tiles gw, gw + GW, ...
  const int w_first = GW - 1 - gw;                                 // window tiles go to the last wavefronts (gw < GW)
  const int n_w = Tw > w_first ? fa_div(Tw - w_first + GW - 1, GW) : 0;

  for (int it = 0; it < n_c + n_w; ++it) {
    const bool win = it >= n_c;
    const int tile = win ? w_first + (it - n_c) * GW : gw + it * GW;
    const int limit = win ? nw : S;             // keys of this region
    const int kbase = tile * 32;
    // ---- S^T = K Q^T ----
    const bf16_t* kp;
    {
      const int key = min(kbase + kperm, limit - 1);
      if (win) {
        kp = k_win + ((size_t)(row0 + key) * Hkv + kvh) * D;
      } else {
        // a lane whose key lies beyond seq_len reads some valid row; its score is replaced below
        const int page = min(max(page_k, 0), g.n_pages - 1);
        kp = k_pages + (((size_t)page * Hkv + kvh) * ps + (kbase + kperm) % ps) * D;
      }
    }
    uint4 kf[8];
#pragma unroll
    for (int ds = 0; ds < 8; ++ds) kf[ds] = (COH && win) ? ld16_coh(kp + ds * 16 + 8 * h) : *(const uint4*)(kp + ds * 16 + 8 * h);
    // ---- V^T fragments: [dt][j]: d = dt*32 + c, keys kbase + 16 j + 8 h .. +8 ----
    uint4 vf[4][2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int key0 = kbase + 16 * j + 8 * h;
      const int nv = limit - key0;
      const bf16_t* vp;
      size_t dstride;
      if (win) {
        vp = vT_win + ((size_t)(n * Hkv + kvh) * D + c) * wpad + min(key0, wpad - 8);
        dstride = (size_t)32 * wpad;
      } else {
        const int page = min(max(page_v[j], 0), g.n_pages - 1);
        vp = v_pages + (((size_t)page * Hkv + kvh) * D + c) * ps + (key0 % ps);
        dstride = (size_t)32 * ps;
      }
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
        vf[dt][j] = mask_keys((COH && win) ? ld16_coh(vp + dt * dstride) : *(const uint4*)(vp + dt * dstride), nv);
    }
    if (it + 1 < n_c) {  // page-table entries of the next cached tile, in flight during this tile's math
      const int nb = (tile + GW) * 32;
      page_k = pt[min(nb + kperm, cap - 1) / ps];
#pragma unroll
      for (int j = 0; j < 2; ++j) page_v[j] = pt[min(nb + 16 * j + 8 * h, cap - 1) / ps];
    }
    f32x16_t sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
    for (int ds = 0; ds < 8; ++ds) {
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[ds]), __builtin_bit_cast(bf16x8_t, qf[ds]), sacc, 0, 0, 0);
      if (SPLIT) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kf[ds]), __builtin_bit_cast(bf16x8_t, ql[ds]), sacc, 0, 0, 0);
    }
    // sacc[i]: key kbase + 16 (i / 8) + 8 h + (i % 8), query row c
    float sv[16];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = kbase + 16 * (i >> 3) + 8 * h + (i & 7);
      bool ok = key < limit;
      if (win) {
        const int w = row0 + key;
        ok = ok && ((w >= lo && w < hi) || w == r);
      }
      sv[i] = ok ? sacc[i] * scale_log2e : -INFINITY;
      mx = fmaxf(mx, sv[i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // no divergent control flow around the MFMAs: a query row that sees nothing yet keeps m = -inf
    // and uses 0 as the reference, which makes every p below exp2(-inf) = 0
    const float m_new = fmaxf(st.m, mx);
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_ref);
    float ls = 0.f;
    bf16x8_t pb[2], pl[SPLIT ? 2 : 1];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float pv = __builtin_amdgcn_exp2f(sv[i] - m_ref);
      ls += pv;
      const __bf16 ph = (__bf16)pv;
      pb[i >> 3][i & 7] = ph;
      if (SPLIT) pl[i >> 3][i & 7] = (__bf16)(pv - (float)ph);
    }
    ls += __shfl_xor(ls, 32, 64);
    st.l = st.l * alpha + ls;
    st.m = m_new;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) st.o[dt][i] *= alpha;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf[dt][j]), pb[j], st.o[dt], 0, 0, 0);
        if (SPLIT) st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vf[dt][j]), pl[j], st.o[dt], 0, 0, 0);
      }
    }
  }
  if (st.l == 12345.678f) return;
  S2D2_ATS(2);
  // ---- merge the wavefronts of the workgroup through LDS, in wavefront order, with all threads ----
  // Every wavefront deposits its state; thread (w, c) of the first NW*32 threads turns the running maxima
  // into per-(wavefront, query row) scale factors; then every thread merges 8 output elements over the NW
  // states.  Element index idx = (dt*4 + i4)*64 + lane holds the 4 consecutive head-dim positions
  // d0 = dt*32 + 8*i4 + 4*h of query row c (lane = 32*h + c): the same order as the MFMA accumulators.
  float* s_o = smem;                              // [NW][16][64] float4
  float* s_m = smem + (size_t)NW * 4096;          // [NW][32]
  float* s_l = s_m + NW * 32;                     // [NW][32]
  float* s_f = s_l + NW * 32;                     // [NW][32] scale of wavefront w for row c
  float* s_ML = s_f + NW * 32;                    // [2][32]  merged max and sum
  {
    float4* dst = (float4*)(s_o + (size_t)wave * 4096) + lane;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        dst[(dt * 4 + i4) * 64] = make_float4(st.o[dt][4 * i4], st.o[dt][4 * i4 + 1], st.o[dt][4 * i4 + 2], st.o[dt][4 * i4 + 3]);
    if (h == 0) { s_m[wave * 32 + c] = st.m; s_l[wave * 32 + c] = st.l; }
  }
  __syncthreads();
  if (threadIdx.x < NW * 32) {
    const int w = threadIdx.x >> 5, cc = threadIdx.x & 31;
    float M = -INFINITY;
#pragma unroll
    for (int w2 = 0; w2 < NW; ++w2) M = fmaxf(M, s_m[w2 * 32 + cc]);
    const float mw = s_m[w * 32 + cc];
    s_f[w * 32 + cc] = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - M);
    if (w == 0) {
      float L = 0.f;
#pragma unroll
      for (int w2 = 0; w2 < NW; ++w2) {   // wavefront order
        const float m2 = s_m[w2 * 32 + cc];
        L += m2 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - M) * s_l[w2 * 32 + cc];
      }
      s_ML[cc] = M;
      s_ML[32 + cc] = L;
    }
  }
  __syncthreads();
  S2D2_ATS(3);
  const int group = item_zy * q_tiles + qt;
  const size_t item0 = (size_t)group * Z;
  constexpr int PER = 16 * 64 / (NW * 64);        // output elements (float4) per thread
#pragma unroll
  for (int k = 0; k < PER; ++k) {
    const int idx = threadIdx.x + k * NW * 64, ln = idx & 63, g16 = idx >> 6, cc = ln & 31, hh = ln >> 5;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int w2 = 0; w2 < NW; ++w2) {
      const float f = s_f[w2 * 32 + cc];
      const float4 v = ((const float4*)(s_o + (size_t)w2 * 4096))[g16 * 64 + ln];
      acc.x += f * v.x; acc.y += f * v.y; acc.z += f * v.z; acc.w += f * v.w;
    }
    if (Zeff == 1) {
      const int qi2 = q0 + cc;
      if (qi2 < nq) {
        const float L = s_ML[32 + cc], inv = L > 0.f ? 1.0f / L : 0.f;
        const int r2 = row0 + qi2 / grp, head2 = kvh * grp + qi2 % grp;
        const int d0 = (g16 >> 2) * 32 + 8 * (g16 & 3) + 4 * hh;
        fa_store4<COH>(o + (size_t)r2 * o_ld + head2 * D + d0, o_lo, acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
      }
    } else {
      st16f_coh(part_o + (item0 + z) * 32 * D + (size_t)idx * 4, acc.x, acc.y, acc.z, acc.w);
    }
  }
  if (Zeff == 1) return;
  // Zeff > 1: this split's partial is written; the workgroup that arrives last merges all splits in split
  // order (so the result does not depend on which one it is) and re-arms the counter.
  if (threadIdx.x < 32) {
    st4f_coh(&part_ml[(item0 + z) * 64 + threadIdx.x], s_ML[threadIdx.x]);
    st4f_coh(&part_ml[(item0 + z) * 64 + 32 + threadIdx.x], s_ML[32 + threadIdx.x]);
  }
  __builtin_amdgcn_s_waitcnt(0);  // the write-through stores of the partial have completed before the arrival is counted
  __syncthreads();
  S2D2_ATS(4);
  int* s_last = (int*)(s_ML + 64);
  if (threadIdx.x == 0) {
    const int prev = __hip_atomic_fetch_add(&counters[group], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_last = prev == Zeff - 1;
    if (prev == Zeff - 1) __hip_atomic_store(&counters[group], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  S2D2_ATS(5);
  if (!*s_last) return;
  S2D2_ATS_ANY(6);
  fa_combine<COH, NW * 64>(part_o, part_ml, item0, Zeff, threadIdx.x, qt, nq, grp, row0, kvh, Hq, o, o_ld, o_lo);
  __builtin_amdgcn_s_waitcnt(0);
  S2D2_ATS_ANY(7);
}


static constexpr size_t fa_lds(int nw) { return ((size_t)nw * (4096 + 96) + 64 + 4) * sizeof(float); }

}  // namespace s2d2
