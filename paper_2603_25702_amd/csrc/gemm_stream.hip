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
// combined through LDS in a fixed order (deterministic).  RMSNorm is folded into the GEMMs on
// both sides of it (see below).  Fused epilogues: fp32 store (logits), residual add (+ operand and
// partial sums of squares of the next norm), SwiGLU, and RoPE + q/k/v split.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

#include <stdlib.h>
#include <string.h>

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

// to_f16: the packed copy holds IEEE half values (the caller's bf16 weights converted; see LO_F16).
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t v) {
  return (uint32_t)f32_to_f16_bits(bf16_to_f32((bf16_t)(v & 0xffffu))) | ((uint32_t)f32_to_f16_bits(bf16_to_f32((bf16_t)(v >> 16))) << 16);
}

__global__ __launch_bounds__(256) void pack_weight_kernel(const bf16_t* __restrict__ W, int N, int K, int NT, int KT,
                                                          int rope_pairs, int D, uint4* __restrict__ out, int to_f16) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)NT * KT * 64) return;
  const int lane = (int)(idx & 63);
  const size_t tile = idx >> 6;
  const int kt = (int)(tile % KT), nt = (int)(tile / KT);
  const int row = packed_row(nt, lane & 15, rope_pairs, D);
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < N) v = *(const uint4*)(W + (size_t)row * K + kt * 32 + (lane >> 4) * 8);
  if (to_f16) v = make_uint4(bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w));
  out[idx] = v;
}

size_t packed_weight_bytes(int N, int K) { return (size_t)((N + 15) / 16) * (K / 32) * 1024; }

void launch_pack_weight(hipStream_t st, const void* W, int N, int K, int rope_pairs, int D, void* out, int to_f16) {
  const int NT = (N + 15) / 16, KT = K / 32;
  const size_t total = (size_t)NT * KT * 64;
  S2D2_LAUNCH(pack_weight_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t*)W, N,
                     K, NT, KT, rope_pairs, D, (uint4*)out, to_f16);
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
  S2D2_LAUNCH(rope_table_kernel, dim3(rows_cap), dim3(64), 0, st, p, D / 2, D, theta, (float2*)cs);
}

// ---------------------------------------------------------------------------------------------
// Latency matters as much as bandwidth here (a layer's matrices are 8-50 MB, a few microseconds
// of HBM time each), so every global load of a wavefront is in flight at once: its weight
// fragments first (they depend on nothing), then the row count, the activation fragments and
// the partial sums of squares.
//
// RMSNorm is split across the producer / consumer pair so that no workgroup has to see a whole
// residual row twice: the residual-add epilogue (SEPI_ADD_F32) of the producing GEMM also writes
// xg = bf16(h * gain_of_the_next_norm) and, per (row, 16-feature tile), the sum of squares of
// its h values; the consuming GEMM (SPRO_BF16S) multiplies xg as it is and scales its fp32 result
// by 1/rms, which it gets by adding the row's partial sums in tile order (deterministic).
template <int NW, int TA>
__device__ __forceinline__ float tile_total(const float* s_red, int t, int fe, int row) {
  const int src = (fe & 3) * 64 + (fe >> 2) * 16 + row;
  float v = 0.f;
#pragma unroll
  for (int w_ = 0; w_ < NW; ++w_) v += s_red[((size_t)w_ * TA + t) * 256 + src];
  return v;
}

#ifdef S2D2_KERNEL_TIMING
__device__ unsigned long long g_stream_ts[4][16];   // [epilogue kind][first workgroup: 0-7, last workgroup: 8-15]
// stamps are kept in registers and written once at the end: a store in the middle of the kernel would turn the
// scalar loads after it into vector loads (possible aliasing) and so change what is being timed
#define S2D2_GTS(k) do { ts_[(k)] = wall_clock64(); } while (0)
#else
#define S2D2_GTS(k) do {} while (0)
#endif

// PAIR (residual-add epilogue, one feature tile per workgroup): K is shared by the 2 NW wavefronts of TWO workgroups,
// so that a matrix with few feature tiles (d_model / 16 of them for the down projection) still puts a workgroup
// on every compute unit.  The workgroups x < gridDim.x / 2 ("producers", dispatched first) reduce their NW shares
// and hand the 16 x 16 partial over as 64-bit (value, tag) words; the workgroup x + gridDim.x / 2 adds its own NW
// shares, waits for those words with a bounded spin, adds them (own + partner: a fixed order), clears them for
// the next launch and runs the epilogue.  Every wait ends: the producers never wait and are resident before
// their consumers; a spin that runs out sets *pair_status and continues with what it has.
template <int EPI, int PRO, int NW, int TPW, int U, int OPM, bool PAIR = false>
__global__ __launch_bounds__(NW * 64) void gemm_stream_kernel(const GemmStreamArgs a) {
  static_assert(!PAIR || (EPI == SEPI_ADD_F32 && TPW == 1), "the paired K split exists for the residual-add epilogue only");
  static_assert(NW >= 4, "the epilogue maps 256 threads onto the 16 x 16 tile (row = thread / 16, feature = thread % 16)");
  constexpr int NACC = EPI == SEPI_SWIGLU ? 2 : 1;
  constexpr int TA = TPW * NACC;
  constexpr bool SPLIT = OPM == OPM_BF16X2;   // the activations come as two bf16 planes
  extern __shared__ __align__(16) uint8_t smem_raw[];
#ifdef S2D2_KERNEL_TIMING
  unsigned long long ts_[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#endif
  S2D2_GTS(0);
  const int m0 = blockIdx.y * 16;
  int M = 0;
  if (blockIdx.y != 0) {  // further row tiles exist only for wide windows: do not stream weights for nothing
    M = *a.m_count;
    if (m0 >= M) return;
  }
  const int nx = PAIR ? (int)gridDim.x / 2 : (int)gridDim.x;
  const bool producer = PAIR && (int)blockIdx.x < nx;
  const int bx = PAIR ? (int)blockIdx.x % nx : (int)blockIdx.x;
  const int nt0 = bx * TPW;
  // The wavefront index is made a scalar: every bound of the K loop derives from it, and a matrix instruction
  // ignores the execution mask.  With the index left in a vector register the `if (kt0 + u < kt_end) mac(u)` of a
  // share's last batch compiles to an execution-mask region, and when that region holds nothing but MFMAs the
  // compiler drops the branch around it: the MFMAs of slots past the share then run with an empty mask and add
  // the (clamped, duplicated) last tile again.  Scalar bounds give scalar branches, which skip the instructions.
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = lane >> 4, f = lane & 15;
  const int KT = a.KT;

  float* s_rs = (float*)smem_raw;                                   // [16] 1/rms per row (SPRO_BF16S)
  float* s_red = s_rs + 16;                                         // [NW][TA][256]

  constexpr int NS = PAIR ? 2 * NW : NW;                            // K shares
  const int share = PAIR ? (producer ? NW : 0) + wave : wave;
  const int kt_begin = (int)((long long)share * KT / NS), kt_end = (int)((long long)(share + 1) * KT / NS);
  const u32x4_t* wp[TA];
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int nt = min(nt0 + t, a.NT - 1);
    wp[t * NACC] = (const u32x4_t*)a.Wp + (size_t)nt * KT * 64 + lane;
    if (NACC == 2) wp[t * NACC + 1] = (const u32x4_t*)a.Wp2 + (size_t)nt * KT * 64 + lane;
  }
  // Loads are unconditional with addresses clamped to the wavefront's share; a slot whose tile lies past the
  // share is never multiplied (uniform test before its MFMAs), and window rows past the row count read row 0:
  // their accumulator rows are never stored.  No select ever sits between a load and its use.
  u32x4_t w[TA][U];
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int t = 0; t < TA; ++t) w[t][u] = ld_stream(&wp[t][(size_t)max(0, min(kt_begin + u, kt_end - 1)) * 64]);

  if (blockIdx.y == 0) M = *a.m_count;
  const int Mloc = min(16, M - m0);
  if (Mloc <= 0) return;  // whole workgroup (M is uniform)

  const bool row_ok = f < Mloc;
  // Row gathering exists for the unembedding only (its rows are the window's logit rows).  Compiled out of the
  // layer GEMMs: the index load would put a wait for ALL earlier loads (the weight stream) in front of the
  // activation loads, also on launches that do not gather.
  constexpr bool CAN_GATHER = EPI == SEPI_STORE_F32;
  const int32_t* gather = CAN_GATHER ? a.gather : nullptr;
  const int xrow_i = m0 + (row_ok ? f : 0);
  const int xrow = gather ? gather[xrow_i] : xrow_i;
  const bf16_t* xg = a.X + (size_t)xrow * a.ldx + g * 8;
  u32x4_t xb[U], xl[SPLIT ? U : 1];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int kc = max(0, min(kt_begin + u, kt_end - 1));   // (an empty share reads tile 0 and multiplies nothing)
    xb[u] = *(const u32x4_t*)(xg + kc * 32);
    if (SPLIT) xl[u] = *(const u32x4_t*)(xg + a.x_lo + kc * 32);
  }

  // 1/rms of the 16 rows from the producer's partial sums of squares: 16 threads per row.  The partials are only
  // REQUESTED here, as independent 16-byte loads (up to four per thread, in flight together with the operand
  // stream); they are added up after the K loop, where the result is first needed.  Reading them one after the
  // other at this point cost eight dependent cache round trips before the first MFMA (5-9 us per launch).
  constexpr int SSV = 4;   // float4 per thread: covers ss_count <= 256, i.e. K <= 4096 (wider: the loop below)
  float4 ssv[SSV];
  const bool ss_vec = PRO == SPRO_BF16S && a.ss_count <= 64 * SSV && (a.ss_count & 3) == 0 && (a.ss_stride & 3) == 0;
  const int ss_row = threadIdx.x >> 4, ss_sub = threadIdx.x & 15;
  const float* ss_pp = nullptr;
  if (PRO == SPRO_BF16S && threadIdx.x < 256) {
    const int rr = m0 + min(ss_row, Mloc - 1);   // rows past the count read a valid row; their 1/rms is never used
    ss_pp = a.ss_part + (size_t)(gather ? gather[rr] : rr) * a.ss_stride;
    if (ss_vec) {
      const int n4 = a.ss_count >> 2;
#pragma unroll
      for (int j = 0; j < SSV; ++j) {
        ssv[j] = ((const float4*)ss_pp)[min(ss_sub + 16 * j, n4 - 1)];   // clamped duplicates are skipped when summing
      }
    }
  }

  f32x4_t acc[TA];
#pragma unroll
  for (int t = 0; t < TA; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  S2D2_GTS(1);
#ifdef S2D2_KERNEL_TIMING
  if (w[0][0][0] == 0x12345678u && Mloc < 0) return;   // (timing aid: the first weight tile has arrived)
  S2D2_GTS(2);
#endif

  // The K loop is a sliding window: register slot u is refilled (weights and activations of the tile U steps on)
  // right after the MFMAs that consumed it have been issued, so a wavefront keeps U tiles in flight continuously
  // instead of loading a batch, draining it, and paying the memory latency again for the next batch.  Whether
  // a batch refills at all is one uniform branch per batch (the last batch of a wavefront's share does not);
  // inside a refilling batch every load is unconditional (addresses clamped to the share), because a load under
  // a per-tile branch, or a select on its result, would make the compiler drain the window first.
  auto mac = [&](int u) {
#pragma unroll
    for (int t = 0; t < TA; ++t) {
      acc[t] = mfma_16x16x32<OPM>(w[t][u], xb[u], acc[t]);
      if (SPLIT)  // low-order plane of the activations: same weights, second product
        acc[t] = mfma_16x16x32<OPM>(w[t][u], xl[u], acc[t]);
    }
  };
  for (int kt0 = kt_begin; kt0 < kt_end; kt0 += U) {
    if (kt0 + U < kt_end) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        mac(u);   // a refilling batch is complete: kt0 + U - 1 < kt_end
        const int kc = max(0, min(kt0 + U + u, kt_end - 1));
#pragma unroll
        for (int t = 0; t < TA; ++t) w[t][u] = ld_stream(&wp[t][(size_t)kc * 64]);
        xb[u] = *(const u32x4_t*)(xg + kc * 32);
        if (SPLIT) xl[u] = *(const u32x4_t*)(xg + a.x_lo + kc * 32);
      }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (kt0 + u < kt_end) mac(u);
    }
  }
  // acc[t][i] = Y[m0 + f][tile t, feature 4 g + i]
#ifdef S2D2_KERNEL_TIMING
  if (acc[0][0] == 12345.678f && Mloc < 0) return;
#endif
  S2D2_GTS(3);
  if (PRO == SPRO_BF16S && threadIdx.x < 256) {
    float v = 0.f;
    if (ss_vec) {
#pragma unroll
      for (int j = 0; j < SSV; ++j)
        if (ss_sub + 16 * j < (a.ss_count >> 2)) v += (ssv[j].x + ssv[j].y) + (ssv[j].z + ssv[j].w);
    } else {
      for (int i = ss_sub; i < a.ss_count; i += 16) v += ss_pp[i];
    }
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 8, 64);
    if (ss_sub == 0) s_rs[ss_row] = 1.0f / sqrtf(v / (float)a.K + a.eps);
  }
#pragma unroll
  for (int t = 0; t < TA; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) s_red[((size_t)wave * TA + t) * 256 + i * 64 + lane] = acc[t][i];
  __syncthreads();
  S2D2_GTS(4);
  if (threadIdx.x >= 256) return;
  const int row = threadIdx.x >> 4, fe = threadIdx.x & 15;
  const int m = m0 + row;
  const bool live = row < Mloc;
  const float rs = PRO == SPRO_BF16S ? s_rs[row] : 1.0f;
#define S2D2_TOTAL(t_, fe_) (tile_total<NW, TA>(s_red, (t_), (fe_), row) * rs)
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int nt = nt0 + t;
    if (nt < a.NT) {
      if (EPI == SEPI_STORE_F32) {
        const int n = nt * 16 + fe;
        if (live && n < a.N) ((float*)a.out)[(size_t)m * a.ldo + n] = S2D2_TOTAL(t, fe);
      } else if (EPI == SEPI_ADD_F32) {
        // residual add; also emits the next norm's operand and this tile's share of the row's sum of squares
        const int n = nt * 16 + fe;
        float hv = 0.f;
        float total = S2D2_TOTAL(t, fe);
        if (PAIR) {
          unsigned long long* slot = a.pair_buf + ((size_t)blockIdx.y * nx + bx) * 256 + threadIdx.x;
          if (producer) {   // (value, tag 1); the store leaves the device-coherent way and the workgroup is done
            __hip_atomic_store(slot, (unsigned long long)__float_as_uint(total) | (1ull << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
          }
          unsigned long long v = 0;
          int spins = 0;
          for (; spins < (1 << 20); ++spins) {
            v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v >> 32) break;
            __builtin_amdgcn_s_sleep(1);
          }
          if (!(v >> 32)) { if (a.pair_status) *a.pair_status = 1; }
          else __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // re-armed for the next launch
          total += __uint_as_float((uint32_t)v);
        }
        if (live && n < a.N) {
          float* hp = (float*)a.out + (size_t)m * a.ldo + n;
          hv = *hp + total;
          *hp = hv;
          if (a.xg_out) act_store1(a.xg_out + (size_t)m * a.xg_ld + n, a.xg_lo, hv * a.gain_next[n]);
        }
        if (a.ss_out) {
          float sq = hv * hv;
          sq += __shfl_xor(sq, 1, 64);
          sq += __shfl_xor(sq, 2, 64);
          sq += __shfl_xor(sq, 4, 64);
          sq += __shfl_xor(sq, 8, 64);
          if (live && fe == 0) a.ss_out[(size_t)m * a.ss_stride + nt] = sq;
        }
      } else if (EPI == SEPI_SWIGLU) {
        const int n = nt * 16 + fe;
        const float gate = S2D2_TOTAL(2 * t, fe), up = S2D2_TOTAL(2 * t + 1, fe);
        if (live && n < a.N) act_store1((bf16_t*)a.out + (size_t)m * a.ldo + n, a.out_lo, gate / (1.0f + __expf(-gate)) * up);
      } else if (live && fe < 8) {  // SEPI_QKV_ROPE: lanes fe < 8 own the pair (i, i + D/2) of one head
        const int D = a.D, half = D >> 1, tiles_per_head = D / 16;
        const int head = nt / tiles_per_head, i = 8 * (nt % tiles_per_head) + fe;
        const float x1 = S2D2_TOTAL(t, fe), x2 = S2D2_TOTAL(t, fe + 8);
        if (head < a.Hq + a.Hkv) {
          const float2 cs = a.rope_cs[(size_t)m * half + i];
          const float y1 = x1 * cs.x - x2 * cs.y, y2 = x2 * cs.x + x1 * cs.y;
          if (head < a.Hq) {  // queries: both planes when the attention kernel multiplies with both
            bf16_t* dst = a.q_out + (size_t)m * a.q_ld + head * D;
            act_store1(dst + i, a.q_lo, y1);
            act_store1(dst + i + half, a.q_lo, y2);
          } else {
            const size_t ko = ((size_t)m * a.Hkv + (head - a.Hq)) * D;
            a.k_out[ko + i] = f32_to_bf16(y1);
            a.k_out[ko + i + half] = f32_to_bf16(y2);
            if (a.k16_out) { a.k16_out[ko + i] = f32_to_f16_bits(y1); a.k16_out[ko + i + half] = f32_to_f16_bits(y2); }
          }
        } else {
          const int vh = head - a.Hq - a.Hkv;
          const bf16_t b1 = f32_to_bf16(x1), b2 = f32_to_bf16(x2);
          bf16_t* dst = a.v_out + ((size_t)m * a.Hkv + vh) * D;
          dst[i] = b1;
          dst[i + half] = b2;
          if (a.vT_out) {  // key-minor copy of the window's V: [seq, Hkv, D, wpad]
            const int n = a.row_seq[m], tw = m - a.seq_row0[n];
            bf16_t* vt = a.vT_out + ((size_t)(n * a.Hkv + vh) * D) * a.wpad + tw;
            vt[(size_t)i * a.wpad] = a.win_f16 ? f32_to_f16_bits(x1) : b1;
            vt[(size_t)(i + half) * a.wpad] = a.win_f16 ? f32_to_f16_bits(x2) : b2;
          }
        }
      }
    }
  }
#undef S2D2_TOTAL
#ifdef S2D2_KERNEL_TIMING
  __builtin_amdgcn_s_waitcnt(0);
  S2D2_GTS(5);
  if (threadIdx.x == 0 && blockIdx.y == 0 && (blockIdx.x == 0 || blockIdx.x == gridDim.x - 1))
    for (int k = 0; k < 6; ++k) g_stream_ts[EPI][(blockIdx.x == 0 ? 0 : 8) + k] = ts_[k];
#endif
}

#ifdef S2D2_KERNEL_TIMING
__global__ void stream_ts_copy_kernel(unsigned long long* out) { if (threadIdx.x < 64) out[threadIdx.x] = (&g_stream_ts[0][0])[threadIdx.x]; }
void launch_stream_ts_copy(hipStream_t st, void* out) { S2D2_LAUNCH(stream_ts_copy_kernel, dim3(1), dim3(64), 0, st, (unsigned long long*)out); }
#else
void launch_stream_ts_copy(hipStream_t, void*) {}
#endif

template <int EPI, int PRO, int NW, int TPW, int U, int OPM>
static void launch_cfg(hipStream_t st, const GemmStreamArgs& a, int m_cap) {
  constexpr int TA = TPW * (EPI == SEPI_SWIGLU ? 2 : 1);
  const size_t lds = 16 * sizeof(float) + (size_t)NW * TA * 256 * sizeof(float);
  dim3 grid((a.NT + TPW - 1) / TPW, (m_cap + 15) / 16), block(NW * 64);
  S2D2_LAUNCH((gemm_stream_kernel<EPI, PRO, NW, TPW, U, OPM>), grid, block, lds, st, a);
}

// residual-add GEMM with K shared by pairs of workgroups (see the kernel's comment): 2 NT workgroups of NW wavefronts
template <int NW, int U, int OPM>
static void launch_pair(hipStream_t st, const GemmStreamArgs& a, int m_cap) {
  const size_t lds = 16 * sizeof(float) + (size_t)NW * 256 * sizeof(float);
  dim3 grid(2 * a.NT, (m_cap + 15) / 16), block(NW * 64);
  S2D2_LAUNCH((gemm_stream_kernel<SEPI_ADD_F32, SPRO_BF16, NW, 1, U, OPM, true>), grid, block, lds, st, a);
}

// Launch shapes (wavefronts per workgroup, feature tiles per workgroup, loads in flight per wavefront), tuned on the
// 1.7B shape: the layer matrices want >= 256 workgroups; with the sliding-window K loop the step time moved by less
// than 2 % over twenty shapes, so one shape per kind is compiled, and each is compared with the CPU reference by the
// parity tests (also on K shares that end in a partial batch of loads).
// The down projection has only d_model / 16 feature tiles (128 for the 1.7B shape): there K is shared by pairs of
// workgroups (256 workgroups: 9.6 us per launch against 13.0 us with 128 workgroups of 16 wavefronts, which
// streamed at half the rate of the other layer GEMMs).
void launch_gemm_stream(hipStream_t st, int kind, const GemmStreamArgs& a, int m_cap) {
  // wide windows: the LDS-tiled kernel reads the weights once per 128 rows instead of once per 16.  Not for a matrix
  // of a few feature tiles (the MoE router, 64 experts): its weights stay in L2, a 256-column tile would be mostly
  // empty, and a row tile of 16 per workgroup spreads the rows over the whole chip.
  if (m_cap > 32 && !(kind == SEPI_STORE_F32 && a.NT <= 8 && !a.gather)) {
    launch_gemm_tile(st, kind, kind == SEPI_ADD_F32 ? SPRO_BF16 : SPRO_BF16S, a, (m_cap + 127) / 128);
    return;
  }
  const int opm = operand_mode(a.x_lo);
#define S2D2_CFG(EPI, PRO, NW, TPW, U)                                                     \
  do {                                                                                     \
    if (opm == OPM_F16) launch_cfg<EPI, PRO, NW, TPW, U, OPM_F16>(st, a, m_cap);           \
    else if (opm == OPM_BF16X2) launch_cfg<EPI, PRO, NW, TPW, U, OPM_BF16X2>(st, a, m_cap); \
    else launch_cfg<EPI, PRO, NW, TPW, U, OPM_BF16>(st, a, m_cap);                         \
  } while (0)
  switch (kind) {
    case SEPI_QKV_ROPE:   // 8 wavefronts x 4 loads in flight (1.8 % over 4 x 8 once the weight loads were non-temporal)
      if (a.NT >= 1024) S2D2_CFG(SEPI_QKV_ROPE, SPRO_BF16S, 4, 2, 4);
      else S2D2_CFG(SEPI_QKV_ROPE, SPRO_BF16S, 8, 1, 4);
      break;
    case SEPI_ADD_F32:
      // long K and few feature tiles (the down projection): pairs of workgroups share K, one workgroup per CU
      if (a.KT >= 128 && a.pair_buf && (long long)a.NT * ((m_cap + 15) / 16) <= a.pair_cap) {
        if (opm == OPM_F16) launch_pair<8, 4, OPM_F16>(st, a, m_cap);   // (16 wavefronts, or 3 to 12 loads in flight: within 1 %)
        else if (opm == OPM_BF16X2) launch_pair<8, 4, OPM_BF16X2>(st, a, m_cap);
        else launch_pair<8, 4, OPM_BF16>(st, a, m_cap);
      } else if (a.KT >= 128) {
        S2D2_CFG(SEPI_ADD_F32, SPRO_BF16, 16, 1, 4);
      } else {   // short K (the output projection): 0.25 % of the 1.7B step over 16 x 4
        S2D2_CFG(SEPI_ADD_F32, SPRO_BF16, 8, 1, 4);
      }
      break;
    case SEPI_SWIGLU:     // 4 x 4: half the wavefronts per feature tile to merge (0.4 % over 8 x 4 with the weights read ahead)
      S2D2_CFG(SEPI_SWIGLU, SPRO_BF16S, 4, 1, 4);
      break;
    case SEPI_STORE_F32:
      S2D2_CFG(SEPI_STORE_F32, SPRO_BF16S, 4, 2, 4);
      break;
  }
#undef S2D2_CFG
}

// First norm of the forward: xg = bf16(h * gain), one partial sum of squares per row; and the row's RoPE table
// (cos / sin of pos * theta^(-2i/D), fp64 phase) when cs is given, which saves the launch of rope_table_kernel.
__global__ __launch_bounds__(256) void embed_norm_kernel(const bf16_t* __restrict__ embed, int d, Plan p,
                                                         const float* __restrict__ gain, float* __restrict__ h,
                                                         bf16_t* __restrict__ xg, int xg_ld, int xg_lo,
                                                         float* __restrict__ ss, int ss_stride,
                                                         float2* __restrict__ cs, int D, float theta) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  if (r >= p.counts[0]) return;
  if (cs) {
    const double pos = (double)p.row_pos[r];
    const int half = D >> 1;
    for (int i = threadIdx.x; i < half; i += 256) {
      const double inv = exp2(-2.0 * (double)i / (double)D * log2((double)theta));
      double sn, c;
      sincos(pos * inv, &sn, &c);
      cs[(size_t)r * half + i] = make_float2((float)c, (float)sn);
    }
  }
  const bf16_t* src = embed + (size_t)p.row_token[r] * d;
  float acc = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float v = bf16_to_f32(src[i]);
    h[(size_t)r * d + i] = v;
    act_store1(xg + (size_t)r * xg_ld + i, xg_lo, v * gain[i]);
    acc += v * v;
  }
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) ss[(size_t)r * ss_stride] = (red[0] + red[1]) + (red[2] + red[3]);
}

void launch_embed_norm(hipStream_t st, const void* embed, int d, const Plan& p, int rows_cap, const float* gain,
                       float* h, void* xg, int xg_ld, int xg_lo, float* ss, int ss_stride, void* rope_cs, int D, float theta) {
  S2D2_LAUNCH(embed_norm_kernel, dim3(rows_cap), dim3(256), 0, st, (const bf16_t*)embed, d, p, gain, h,
                     (bf16_t*)xg, xg_ld, xg_lo, ss, ss_stride, (float2*)rope_cs, D, theta);
}

}  // namespace s2d2
