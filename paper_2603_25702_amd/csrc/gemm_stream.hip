// Weight-streaming GEMM for the decode regime on packed bf16 weights, with the row-wise work of
// the decoder fused in:  Y[m, n] = sum_k X[m, k] W[n, k],  M <= 16 rows per row tile.
//
// Packed layout (built once by pack_weight_kernel): the matrix is cut into tiles of 16 output
// features x 32 inputs; a tile is stored as 64 lanes x 16 bytes in exactly the register order
// of the A operand of v_mfma_f32_16x16x32_bf16 (lane l holds row l%16, inputs 8*(l/16)..+7).
// One wavefront-wide 16-byte load therefore reads 1 KB of contiguous memory and is a complete
// MFMA operand: no LDS and no shuffles on the weight path, fully coalesced HBM reads.
//
// A workgroup owns TPW feature tiles; its NW wavefronts split K into contiguous ranges and are
// combined through LDS in a fixed order (deterministic).  Fused prologue: RMSNorm of the fp32
// residual rows (gain applied before the bf16 rounding, 1/rms applied to the fp32 result).
// Fused epilogues: fp32 store (logits), residual add, SwiGLU, and RoPE + q/k/v split.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

namespace s2d2 {

// ---------------------------------------------------------------------------------------------
// Packing.  rope_pairs != 0 (the fused QKV matrix): tile j of a head holds the rows
// {8j..8j+7} and {D/2+8j..D/2+8j+7} of that head, so a rotation pair lives in one tile.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int packed_row(int nt, int f, int rope_pairs, int D) {
  if (!rope_pairs) return nt * 16 + f;
  const int tiles_per_head = D / 16;
  const int head = nt / tiles_per_head, j = nt % tiles_per_head;
  return head * D + (f < 8 ? 8 * j + f : D / 2 + 8 * j + (f - 8));
}

__global__ __launch_bounds__(256) void pack_weight_kernel(const bf16_t* __restrict__ W, int N, int K, int NT, int KT,
                                                          int rope_pairs, int D, uint4* __restrict__ out) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)NT * KT * 64) return;
  const int lane = (int)(idx & 63);
  const size_t tile = idx >> 6;
  const int kt = (int)(tile % KT), nt = (int)(tile / KT);
  const int row = packed_row(nt, lane & 15, rope_pairs, D);
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < N) v = *(const uint4*)(W + (size_t)row * K + kt * 32 + (lane >> 4) * 8);
  out[idx] = v;
}

size_t packed_weight_bytes(int N, int K) { return (size_t)((N + 15) / 16) * (K / 32) * 1024; }

void launch_pack_weight(hipStream_t st, const void* W, int N, int K, int rope_pairs, int D, void* out) {
  const int NT = (N + 15) / 16, KT = K / 32;
  const size_t total = (size_t)NT * KT * 64;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t*)W, N,
                     K, NT, KT, rope_pairs, D, (uint4*)out);
}

// cos / sin of pos * theta^(-2i/D) for every window row (fp64 phase), [rows, D/2] float2
__global__ void rope_table_kernel(Plan p, int half, int D, float theta, float2* __restrict__ cs) {
  const int r = blockIdx.x;
  if (r >= p.counts[0]) return;
  const double pos = (double)p.row_pos[r];
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double inv = exp2(-2.0 * (double)i / (double)D * log2((double)theta));
    double s, c;
    sincos(pos * inv, &s, &c);
    cs[(size_t)r * half + i] = make_float2((float)c, (float)s);
  }
}

void launch_rope_table(hipStream_t st, const Plan& p, int rows_cap, int D, float theta, void* cs) {
  hipLaunchKernelGGL(rope_table_kernel, dim3(rows_cap), dim3(64), 0, st, p, D / 2, D, theta, (float2*)cs);
}

// ---------------------------------------------------------------------------------------------
// Latency matters as much as bandwidth here (a layer's matrices are 8-50 MB, a few microseconds
// of HBM time each), so the kernel is arranged to have every global load in flight at once:
// the wavefront's weight fragments are requested first (they depend on nothing), then the row
// count, then all residual rows of the fused RMSNorm (one column group per thread, all rows
// unrolled), and only then does anything wait.
template <int NW, int TA>
__device__ __forceinline__ float tile_total(const float* s_red, int t, int fe, int row) {
  const int src = (fe & 3) * 64 + (fe >> 2) * 16 + row;
  float v = 0.f;
#pragma unroll
  for (int w_ = 0; w_ < NW; ++w_) v += s_red[((size_t)w_ * TA + t) * 256 + src];
  return v;
}

template <int EPI, int PRO, int NW, int TPW, int U>
__global__ __launch_bounds__(NW * 64) void gemm_stream_kernel(const GemmStreamArgs a) {
  constexpr int NACC = EPI == SEPI_SWIGLU ? 2 : 1;
  constexpr int TA = TPW * NACC;
  constexpr int T = NW * 64;
  extern __shared__ __align__(16) uint8_t smem_raw[];
  const int m0 = blockIdx.y * 16;
  int M = 0;
  if (blockIdx.y != 0) {  // further row tiles exist only for wide windows: do not stream weights for nothing
    M = *a.m_count;
    if (m0 >= M) return;
  }
  const int nt0 = blockIdx.x * TPW;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, f = lane & 15;
  const int K = a.K, KT = a.KT;
  const int xs_stride = K + 8;  // bf16 elements; 16-byte skew between rows avoids LDS bank conflicts

  float* s_part = (float*)smem_raw;                                 // [NW][16] partial sums of squares
  float* s_red = s_part + NW * 16;                                  // [NW][TA][256]
  bf16_t* xs = (bf16_t*)(s_red + (size_t)NW * TA * 256);            // [16][K + 8] (SPRO_NORM only)

  const u32x4_t zero = {0u, 0u, 0u, 0u};
  const int kt_begin = (int)((long long)wave * KT / NW), kt_end = (int)((long long)(wave + 1) * KT / NW);
  const u32x4_t* wp[TA];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int nt = min(nt0 + t, a.NT - 1);
    wp[t * NACC] = (const u32x4_t*)a.Wp + (size_t)nt * KT * 64 + lane;
    if (NACC == 2) wp[t * NACC + 1] = (const u32x4_t*)a.Wp2 + (size_t)nt * KT * 64 + lane;
  }
  u32x4_t w[TA][U];
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int t = 0; t < TA; ++t) w[t][u] = (kt_begin + u < kt_end) ? wp[t][(size_t)(kt_begin + u) * 64] : zero;

  if (blockIdx.y == 0) M = *a.m_count;
  const int Mloc = min(16, M - m0);
  if (Mloc <= 0) return;  // whole workgroup (M is uniform)

  if (PRO == SPRO_NORM) {
    // thread -> group of 4 columns, all rows: Mloc + 1 independent 16-byte loads per group
    const int C4 = K >> 2;
    float ss[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) ss[r] = 0.f;
    for (int c = threadIdx.x; c < C4; c += T) {
      const f32x4_t gn = ((const f32x4_t*)a.gain)[c];
      f32x4_t hv[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (r < Mloc) {
          const int src = a.gather ? a.gather[m0 + r] : m0 + r;
          hv[r] = ((const f32x4_t*)a.H)[(size_t)src * C4 + c];
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        u32x2_t pk = {0u, 0u};
        if (r < Mloc) {
          const f32x4_t h = hv[r];
          ss[r] += h.x * h.x + h.y * h.y + h.z * h.z + h.w * h.w;
          pk.x = (uint32_t)f32_to_bf16(h.x * gn.x) | ((uint32_t)f32_to_bf16(h.y * gn.y) << 16);
          pk.y = (uint32_t)f32_to_bf16(h.z * gn.z) | ((uint32_t)f32_to_bf16(h.w * gn.w) << 16);
        }
        *(u32x2_t*)(xs + (size_t)r * xs_stride + 4 * c) = pk;
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if (r < Mloc) {
        float v = ss[r];
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == 0) s_part[wave * 16 + r] = v;
      }
    }
    __syncthreads();
  }

  f32x4_t acc[TA];
#pragma unroll
  for (int t = 0; t < TA; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const bool row_ok = f < Mloc;
  const bf16_t* xg = PRO == SPRO_BF16 ? a.X + (size_t)(row_ok ? m0 + f : m0) * a.ldx + g * 8 : nullptr;
  const bf16_t* xl = xs + (size_t)f * xs_stride + g * 8;

  for (int kt0 = kt_begin; kt0 < kt_end;) {
    u32x4_t xb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kt = kt0 + u;
      const bool ok = kt < kt_end;
      if (PRO == SPRO_NORM) xb[u] = ok ? *(const u32x4_t*)(xl + kt * 32) : zero;
      else xb[u] = (ok && row_ok) ? *(const u32x4_t*)(xg + kt * 32) : zero;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < TA; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, w[t][u]),
                                                         __builtin_bit_cast(bf16x8_t, xb[u]), acc[t], 0, 0, 0);
    kt0 += U;
    if (kt0 < kt_end) {  // next batch (the layer matrices are sized so that one batch covers a wavefront's share)
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int t = 0; t < TA; ++t) w[t][u] = (kt0 + u < kt_end) ? wp[t][(size_t)(kt0 + u) * 64] : zero;
    }
  }
  // acc[t][i] = Y[m0 + f][tile t, feature 4 g + i]
#pragma unroll
  for (int t = 0; t < TA; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) s_red[((size_t)wave * TA + t) * 256 + i * 64 + lane] = acc[t][i];
  __syncthreads();
  if (threadIdx.x >= 256) return;
  const int row = threadIdx.x >> 4, fe = threadIdx.x & 15;
  const int m = m0 + row;
  if (row >= Mloc) return;
  float rs = 1.0f;
  if (PRO == SPRO_NORM) {
    float v = 0.f;
#pragma unroll
    for (int w_ = 0; w_ < NW; ++w_) v += s_part[w_ * 16 + row];
    rs = 1.0f / sqrtf(v / (float)K + a.eps);
  }
#define S2D2_TOTAL(t_, fe_) (tile_total<NW, TA>(s_red, (t_), (fe_), row) * rs)
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int nt = nt0 + t;
    if (nt < a.NT) {
      if (EPI == SEPI_STORE_F32) {
        const int n = nt * 16 + fe;
        if (n < a.N) ((float*)a.out)[(size_t)m * a.ldo + n] = S2D2_TOTAL(t, fe);
      } else if (EPI == SEPI_ADD_F32) {
        const int n = nt * 16 + fe;
        if (n < a.N) ((float*)a.out)[(size_t)m * a.ldo + n] += S2D2_TOTAL(t, fe);
      } else if (EPI == SEPI_SWIGLU) {
        const int n = nt * 16 + fe;
        const float gate = S2D2_TOTAL(2 * t, fe), up = S2D2_TOTAL(2 * t + 1, fe);
        if (n < a.N) ((bf16_t*)a.out)[(size_t)m * a.ldo + n] = f32_to_bf16(gate / (1.0f + __expf(-gate)) * up);
      } else if (fe < 8) {  // SEPI_QKV_ROPE: lanes fe < 8 own the pair (i, i + D/2) of one head
        const int D = a.D, half = D >> 1, tiles_per_head = D / 16;
        const int head = nt / tiles_per_head, i = 8 * (nt % tiles_per_head) + fe;
        const float x1 = S2D2_TOTAL(t, fe), x2 = S2D2_TOTAL(t, fe + 8);
        if (head < a.Hq + a.Hkv) {
          const float2 cs = a.rope_cs[(size_t)m * half + i];
          const float y1 = x1 * cs.x - x2 * cs.y, y2 = x2 * cs.x + x1 * cs.y;
          bf16_t* dst = head < a.Hq ? a.q_out + ((size_t)m * a.Hq + head) * D
                                    : a.k_out + ((size_t)m * a.Hkv + (head - a.Hq)) * D;
          dst[i] = f32_to_bf16(y1);
          dst[i + half] = f32_to_bf16(y2);
        } else {
          const int vh = head - a.Hq - a.Hkv;
          const bf16_t b1 = f32_to_bf16(x1), b2 = f32_to_bf16(x2);
          bf16_t* dst = a.v_out + ((size_t)m * a.Hkv + vh) * D;
          dst[i] = b1;
          dst[i + half] = b2;
          if (a.vT_out) {  // key-minor copy of the window's V: [seq, Hkv, D, wpad]
            const int n = a.row_seq[m], tw = m - a.seq_row0[n];
            bf16_t* vt = a.vT_out + ((size_t)(n * a.Hkv + vh) * D) * a.wpad + tw;
            vt[(size_t)i * a.wpad] = b1;
            vt[(size_t)(i + half) * a.wpad] = b2;
          }
        }
      }
    }
  }
}

template <int EPI, int PRO, int NW, int TPW, int U>
static void launch_cfg(hipStream_t st, const GemmStreamArgs& a, int m_cap) {
  constexpr int TA = TPW * (EPI == SEPI_SWIGLU ? 2 : 1);
  size_t lds = (size_t)NW * 16 * sizeof(float) + (size_t)NW * TA * 256 * sizeof(float);
  if (PRO == SPRO_NORM) lds += (size_t)16 * (a.K + 8) * sizeof(bf16_t);
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)gemm_stream_kernel<EPI, PRO, NW, TPW, U>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    attr_set = true;
  }
  dim3 grid((a.NT + TPW - 1) / TPW, (m_cap + 15) / 16), block(NW * 64);
  hipLaunchKernelGGL((gemm_stream_kernel<EPI, PRO, NW, TPW, U>), grid, block, lds, st, a);
}

bool gemm_stream_norm_fits(int K) { return 16 * 16 * sizeof(float) + 16 * 4 * 256 * sizeof(float) + (size_t)16 * (K + 8) * 2 <= 160 * 1024; }

// Launch shapes: the layer matrices want >= 256 workgroups / >= 2000 wavefronts with the whole
// share of a wavefront in one batch of loads; the unembedding is long enough to batch.
void launch_gemm_stream(hipStream_t st, int kind, const GemmStreamArgs& a, int m_cap) {
  switch (kind) {
    case SEPI_QKV_ROPE:
      if (a.NT >= 1024) launch_cfg<SEPI_QKV_ROPE, SPRO_NORM, 4, 2, 4>(st, a, m_cap);
      else launch_cfg<SEPI_QKV_ROPE, SPRO_NORM, 8, 1, 8>(st, a, m_cap);
      break;
    case SEPI_ADD_F32:
      if (a.KT >= 128) launch_cfg<SEPI_ADD_F32, SPRO_BF16, 16, 1, 12>(st, a, m_cap);
      else launch_cfg<SEPI_ADD_F32, SPRO_BF16, 16, 1, 4>(st, a, m_cap);
      break;
    case SEPI_SWIGLU:
      launch_cfg<SEPI_SWIGLU, SPRO_NORM, 8, 1, 8>(st, a, m_cap);
      break;
    case SEPI_STORE_F32:
      launch_cfg<SEPI_STORE_F32, SPRO_NORM, 4, 4, 4>(st, a, m_cap);
      break;
  }
}

}  // namespace s2d2
