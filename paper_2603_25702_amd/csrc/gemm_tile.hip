// LDS-tiled MFMA GEMM on the packed bf16 weights for windows of more than 32 rows:
//   Y[m, n] = sum_k X[m, k] W[n, k]
// (verifier / draft forwards of the batched configurations, the prompt prefill, and the grouped
// expert GEMMs of the MoE FFN).
//
// A workgroup of four wavefronts owns a tile of 128 rows x 128 output features and walks K in
// steps of 64.  The activation tile goes through LDS (double-buffered, rows padded to 144 bytes so
// that the 16-byte operand reads of a wavefront hit 64 distinct banks); the weight operands are
// read straight from the packed copy, where one wavefront-wide 16-byte load is a complete A
// operand of v_mfma_f32_16x16x32_bf16, one step ahead of their use.  Each wavefront computes
// 64 rows x 64 features (4 x 4 MFMA tiles, 8 x 4 for the gate/up pair of SwiGLU).
//
// The prologue / epilogues are the ones of the streaming kernel (same argument block): 1/rms from
// the producer's partial sums of squares, fp32 store, residual add with the operand and partial
// sums of the next norm, SwiGLU, RoPE + q/k/v split.  In grouped mode a row tile belongs to one
// expert: rows are gathered through the expert-sorted slot list and the down projection scatters
// its result, scaled by the routing weight, to the (token, slot) row it came from.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

namespace s2d2 {

static constexpr int TM = 128, TN = 128, TK = 64;

// SPLIT: the activations come as a high- and a low-order bf16 plane (16 significant bits); both planes
// of a row sit side by side in LDS and every weight operand is multiplied with both.
template <int EPI, int PRO, bool SPLIT>
__global__ __launch_bounds__(256) void gemm_tile_kernel(const GemmStreamArgs a) {
  constexpr int NACC = EPI == SEPI_SWIGLU ? 2 : 1;
  constexpr int XROW = (SPLIT ? 256 : 128) + 16;  // bytes per LDS row: 64 bf16 per plane + 16 bytes of padding
  __shared__ __align__(16) uint8_t s_x[2][TM * XROW];
  __shared__ int s_xrow[TM], s_orow[TM];
  __shared__ float s_rs[TM];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 4, f = lane & 15;
  const int wr = wave >> 1, wc = wave & 1;
  int m0, Mloc, expert = 0;
  if (a.grouped != GROUP_NONE) {
    if ((int)blockIdx.y >= *a.n_tiles) return;
    expert = a.tile_expert[blockIdx.y];
    m0 = a.tile_row0[blockIdx.y];
    Mloc = a.tile_rows[blockIdx.y];
  } else {
    const int M = *a.m_count;
    m0 = blockIdx.y * TM;
    if (m0 >= M) return;
    Mloc = min(TM, M - m0);
  }
  const int KT = a.KT;
  const int nt0 = blockIdx.x * (TN / 16) + wc * 4;

  // ---- row maps: source row of X, row of the partial sums of squares, destination row, scale ----
  {
    const int r = tid >> 1, hf = tid & 1;   // two threads per row
    int xrow = -1, orow = -1, ssrow = 0;
    float ow = 1.f;
    if (r < Mloc) {
      const int s = m0 + r;
      if (a.grouped == GROUP_GATHER) {          // expert gate/up: X row of the token, output in sorted order
        xrow = a.sorted[s] / a.top_k; ssrow = xrow; orow = s;
      } else if (a.grouped == GROUP_SCATTER) {  // expert down: X in sorted order, output to the (token, slot) row
        xrow = s; orow = a.sorted[s]; ow = a.route_w[orow];
      } else {
        xrow = a.gather ? a.gather[s] : s; ssrow = xrow; orow = s;
      }
    }
    float rs = ow;
    if (PRO == SPRO_BF16S) {
      float v = 0.f;
      if (r < Mloc) {
        const float* pp = a.ss_part + (size_t)ssrow * a.ss_stride;
        for (int i = hf; i < a.ss_count; i += 2) v += pp[i];
      }
      v += __shfl_xor(v, 1, 64);
      rs *= 1.0f / sqrtf(v / (float)a.K + a.eps);
    }
    if (hf == 0) { s_xrow[r] = xrow; s_orow[r] = orow; s_rs[r] = rs; }
  }
  __syncthreads();

  // ---- operand addressing ----
  const int c16 = tid & 7, rbase = tid >> 3;   // this thread stages rows rbase + 32 i, bytes [16 c16, +16) of the 128
  const bf16_t* xsrc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int xr = s_xrow[rbase + 32 * i];
    xsrc[i] = xr >= 0 ? a.X + (size_t)xr * a.ldx + c16 * 8 : nullptr;
  }
  const u32x4_t* wp[4 * NACC];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int nt = min(nt0 + t, a.NT - 1);
    wp[t * NACC] = (const u32x4_t*)a.Wp + (size_t)expert * a.expert_stride + (size_t)nt * KT * 64 + lane;
    if (NACC == 2) wp[t * NACC + 1] = (const u32x4_t*)a.Wp2 + (size_t)expert * a.expert_stride + (size_t)nt * KT * 64 + lane;
  }
  const u32x4_t zero = {0u, 0u, 0u, 0u};

  f32x4_t acc[4][4 * NACC];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int t = 0; t < 4 * NACC; ++t) acc[rb][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int nk = (a.K + TK - 1) / TK;
  u32x4_t xr[4], xl[SPLIT ? 4 : 1], wn[2][4 * NACC], wcur[2][4 * NACC];
  auto load_x = [&](int kb) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = kb * TK + c16 * 8;
      xr[i] = (xsrc[i] && k < a.K) ? *(const u32x4_t*)(xsrc[i] + kb * TK) : zero;
      if (SPLIT) xl[i] = (xsrc[i] && k < a.K) ? *(const u32x4_t*)(xsrc[i] + a.x_lo + kb * TK) : zero;
    }
  };
  auto load_w = [&](int kb) {
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      const int kt = kb * 2 + k2;
#pragma unroll
      for (int t = 0; t < 4 * NACC; ++t) wn[k2][t] = kt < KT ? wp[t][(size_t)kt * 64] : zero;
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(u32x4_t*)(s_x[buf] + (rbase + 32 * i) * XROW + c16 * 16) = xr[i];
      if (SPLIT) *(u32x4_t*)(s_x[buf] + (rbase + 32 * i) * XROW + 128 + c16 * 16) = xl[i];
    }
  };

  load_x(0);
  load_w(0);
  store_x(0);
  __syncthreads();
  for (int kb = 0; kb < nk; ++kb) {
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
      for (int t = 0; t < 4 * NACC; ++t) wcur[k2][t] = wn[k2][t];
    if (kb + 1 < nk) {
      load_x(kb + 1);
      load_w(kb + 1);
    }
    const uint8_t* xb = s_x[kb & 1] + (wr * 64 + f) * XROW + g * 16;
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        const u32x4_t b = *(const u32x4_t*)(xb + rb * 16 * XROW + k2 * 64);
#pragma unroll
        for (int t = 0; t < 4 * NACC; ++t)
          acc[rb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wcur[k2][t]),
                                                               __builtin_bit_cast(bf16x8_t, b), acc[rb][t], 0, 0, 0);
        if (SPLIT) {
          const u32x4_t bl = *(const u32x4_t*)(xb + rb * 16 * XROW + 128 + k2 * 64);
#pragma unroll
          for (int t = 0; t < 4 * NACC; ++t)
            acc[rb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wcur[k2][t]),
                                                                 __builtin_bit_cast(bf16x8_t, bl), acc[rb][t], 0, 0, 0);
        }
      }
    }
    if (kb + 1 < nk) store_x((kb + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: acc[rb][t][i] = Y[row wr*64 + rb*16 + f][feature (nt0 + t)*16 + 4 g + i] ----
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    const int r = wr * 64 + rb * 16 + f;
    const bool live = r < Mloc;
    const int orow = live ? s_orow[r] : 0;
    const float rs = s_rs[r];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int nt = nt0 + t;
      if (nt >= a.NT) continue;   // uniform over the wavefront
      const int n = nt * 16 + 4 * g;
      if (EPI == SEPI_STORE_F32) {
        if (live) {
          float* op = (float*)a.out + (size_t)orow * a.ldo + n;
          const f32x4_t v = acc[rb][t] * rs;
          if (n + 3 < a.N) *(float4*)op = make_float4(v[0], v[1], v[2], v[3]);
          else
            for (int i = 0; i < 4; ++i)
              if (n + i < a.N) op[i] = v[i];
        }
      } else if (EPI == SEPI_ADD_F32) {
        float hv[4] = {0.f, 0.f, 0.f, 0.f};
        if (live) {
          float* hp = (float*)a.out + (size_t)orow * a.ldo + n;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n + i < a.N) { hv[i] = hp[i] + acc[rb][t][i] * rs; hp[i] = hv[i]; }
          if (a.xg_out) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (n + i < a.N) {
                bf16_t hi, lo;
                split_bf16(hv[i] * a.gain_next[n + i], hi, lo);
                a.xg_out[(size_t)orow * a.xg_ld + n + i] = hi;
                if (a.xg_lo) a.xg_out[(size_t)orow * a.xg_ld + a.xg_lo + n + i] = lo;
              }
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
          bf16_t* op = (bf16_t*)a.out + (size_t)orow * a.ldo + n;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float gate = acc[rb][2 * t][i] * rs, up = acc[rb][2 * t + 1][i] * rs;
            if (n + i < a.N) {
              bf16_t hi, lo;
              split_bf16(gate / (1.0f + __expf(-gate)) * up, hi, lo);
              op[i] = hi;
              if (a.out_lo) op[a.out_lo + i] = lo;
            }
          }
        }
      } else {  // SEPI_QKV_ROPE: features 0-7 of a tile pair with features 8-15 (lanes 32 apart)
        const int D = a.D, half = D >> 1, tiles_per_head = D / 16;
        const int head = nt / tiles_per_head, i0 = 8 * (nt % tiles_per_head) + 4 * (g & 1);
        float own[4], oth[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          own[i] = acc[rb][t][i] * rs;
          oth[i] = __shfl_xor(own[i], 32, 64);
        }
        if (live) {
          const bool second = g >= 2;   // this lane holds x2 (element i + D/2) of the pair
          if (head < a.Hq + a.Hkv) {
            const bool is_q = head < a.Hq;
            bf16_t* dst = is_q ? a.q_out + (size_t)orow * a.q_ld + head * D
                               : a.k_out + ((size_t)orow * a.Hkv + (head - a.Hq)) * D;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float2 cs = a.rope_cs[(size_t)orow * half + i0 + i];
              const float y = second ? own[i] * cs.x + oth[i] * cs.y : own[i] * cs.x - oth[i] * cs.y;
              bf16_t hi, lo;
              split_bf16(y, hi, lo);
              dst[i0 + i + (second ? half : 0)] = hi;
              if (is_q && a.q_lo) dst[a.q_lo + i0 + i + (second ? half : 0)] = lo;
            }
          } else {
            const int vh = head - a.Hq - a.Hkv;
            bf16_t* dst = a.v_out + ((size_t)orow * a.Hkv + vh) * D + (second ? half : 0);
            const int sq = a.row_seq[orow], tw = orow - a.seq_row0[sq];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const bf16_t b = f32_to_bf16(own[i]);
              dst[i0 + i] = b;
              if (a.vT_out)
                a.vT_out[((size_t)(sq * a.Hkv + vh) * D + i0 + i + (second ? half : 0)) * a.wpad + tw] = b;
            }
          }
        }
      }
    }
  }
}

template <int EPI, int PRO>
static void launch_tile(hipStream_t st, const GemmStreamArgs& a, int row_tiles) {
  dim3 grid((a.NT + TN / 16 - 1) / (TN / 16), row_tiles), block(256);
  if (a.x_lo) S2D2_LAUNCH((gemm_tile_kernel<EPI, PRO, true>), grid, block, 0, st, a);
  else S2D2_LAUNCH((gemm_tile_kernel<EPI, PRO, false>), grid, block, 0, st, a);
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
