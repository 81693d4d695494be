// Mixture-of-experts FFN around the grouped tile GEMM: routing, grouping of (token, slot) pairs
// by expert, and the fixed-order combine.
//
//   router logits [rows, E] (fp32, from the GEMM)  ->  softmax over all experts, top-k by value
//   with ties to the lower index, weights renormalised to sum 1 (no shared expert, no capacity
//   limit).  Every (token, slot) pair takes a place in its expert's group through an integer
//   atomic counter in LDS (one workgroup groups all pairs; device-scope atomics from every routing
//   wavefront on E addresses cost 25-40 us per launch); the order inside a group depends on
//   scheduling, but every pair's result is computed from its own row only and written to its own
//   (token, slot) row, and the combine adds the k slots of a token in slot order, so the output is
//   deterministic.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

namespace s2d2 {

static constexpr int MOE_MAX_E = 256;   // experts per lane <= 4

// One wavefront per row.
__global__ __launch_bounds__(256) void moe_route_kernel(const float* __restrict__ logits, int E, int top_k,
                                                        const int32_t* __restrict__ m_count,
                                                        int32_t* __restrict__ choice, float* __restrict__ route_w) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= *m_count) return;
  float v[4];
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = lane + 64 * j;
    v[j] = e < E ? logits[(size_t)row * E + e] : -INFINITY;
    m = fmaxf(m, v[j]);
  }
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  float p[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) p[j] = v[j] > -INFINITY ? __expf(v[j] - m) : 0.f;   // common factor 1/Z cancels in the renormalisation
  // top-k of the logits (softmax is monotone), lowest index on ties
  float wsel = 0.f;      // lane k keeps the k-th selected probability
  int esel = -1;
  float wsum = 0.f;
  for (int k = 0; k < top_k; ++k) {
    float best = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; ++j) best = fmaxf(best, v[j]);
    float bw = best;
    for (int off = 32; off > 0; off >>= 1) bw = fmaxf(bw, __shfl_xor(bw, off, 64));
    int cand = 0x7fffffff;
#pragma unroll
    for (int j = 3; j >= 0; --j)
      if (v[j] == bw) cand = lane + 64 * j;
    int ce = cand;
    for (int off = 32; off > 0; off >>= 1) ce = min(ce, __shfl_xor(ce, off, 64));
    // the owner removes it and publishes its probability
    float pw = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (lane + 64 * j == ce) { pw = p[j]; v[j] = -INFINITY; }
    for (int off = 32; off > 0; off >>= 1) pw += __shfl_xor(pw, off, 64);
    wsum += pw;
    if (lane == k) { wsel = pw; esel = ce; }
  }
  if (lane < top_k) {
    const int o = row * top_k + lane;
    choice[o] = esel;
    route_w[o] = wsel / wsum;
  }
}

// One workgroup: group offsets, the list of 128-row tiles, the expert-sorted slot list; re-arms the counters.
// A thread keeps its slots' choices in registers between the two passes and requests them eight at a time (read one
// per loop iteration, 16 K slots cost 32 dependent L2 round trips per thread); the tile list is written by one thread
// per expert after a scan that touches LDS only.
__global__ __launch_bounds__(1024) void moe_group_kernel(int E, int top_k, const int32_t* __restrict__ m_count,
                                                         const int32_t* __restrict__ choice,
                                                         int32_t* __restrict__ sorted, int32_t* __restrict__ tile_expert,
                                                         int32_t* __restrict__ tile_row0, int32_t* __restrict__ tile_rows,
                                                         int32_t* __restrict__ n_tiles, int tile_cap) {
  __shared__ int s_off[MOE_MAX_E + 1], s_tile0[MOE_MAX_E + 1];
  __shared__ int s_cnt[MOE_MAX_E], s_fill[MOE_MAX_E];
  const int tid = threadIdx.x;
  const int total = *m_count * top_k;
  constexpr int KEEP = 24;   // slots per thread held in registers (24 K slots); the rest is read again in the second pass
  int mine[KEEP];
#pragma unroll
  for (int j0 = 0; j0 < KEEP; j0 += 8) {
#pragma unroll
    for (int j = j0; j < j0 + 8; ++j) mine[j] = (tid + j * 1024 < total) ? choice[tid + j * 1024] : -1;
  }
  for (int e = tid; e < E; e += 1024) { s_cnt[e] = 0; s_fill[e] = 0; }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < KEEP; ++j)
    if (mine[j] >= 0) atomicAdd(&s_cnt[mine[j]], 1);
  for (int i = tid + KEEP * 1024; i < total; i += 1024) atomicAdd(&s_cnt[choice[i]], 1);
  __syncthreads();
  if (tid == 0) {   // offsets of the groups and of their tiles
    int run = 0, t = 0;
    for (int e = 0; e < E; ++e) {
      const int c = s_cnt[e];
      s_off[e] = run;
      s_tile0[e] = t;
      run += c;
      t += (c + 127) >> 7;
    }
    s_off[E] = run;
    s_tile0[E] = t;
    *n_tiles = min(t, tile_cap);
  }
  __syncthreads();
  for (int e = tid; e < E; e += 1024) {
    const int c = s_cnt[e], run = s_off[e];
    int t = s_tile0[e];
    for (int r0 = 0; r0 < c && t < tile_cap; r0 += 128, ++t) {
      tile_expert[t] = e;
      tile_row0[t] = run + r0;
      tile_rows[t] = min(128, c - r0);
    }
  }
#pragma unroll
  for (int j = 0; j < KEEP; ++j)
    if (mine[j] >= 0) sorted[s_off[mine[j]] + atomicAdd(&s_fill[mine[j]], 1)] = tid + j * 1024;
  for (int i = tid + KEEP * 1024; i < total; i += 1024) {
    const int e = choice[i];
    sorted[s_off[e] + atomicAdd(&s_fill[e], 1)] = i;
  }
}

// h[row] += sum over slots (in slot order) of y[row, slot]; also the operand and the partial sums
// of squares of the next norm (one partial per 16 features, like the GEMM epilogue writes them).
__global__ __launch_bounds__(256) void moe_combine_kernel(const float* __restrict__ y, int d, int top_k,
                                                          const int32_t* __restrict__ m_count, float* __restrict__ h,
                                                          bf16_t* __restrict__ xg, int xg_ld, int xg_lo,
                                                          const float* __restrict__ gain_next,
                                                          float* __restrict__ ss, int ss_stride) {
  const int row = blockIdx.x;
  if (row >= *m_count) return;
  for (int c = threadIdx.x * 4; c < d; c += 1024) {
    float4 acc = *(const float4*)(h + (size_t)row * d + c);
    for (int k = 0; k < top_k; ++k) {
      const float4 t = *(const float4*)(y + ((size_t)row * top_k + k) * d + c);
      acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
    }
    *(float4*)(h + (size_t)row * d + c) = acc;
    const float4 gn = *(const float4*)(gain_next + c);
    const float xv[4] = {acc.x * gn.x, acc.y * gn.y, acc.z * gn.z, acc.w * gn.w};
    act_store4(xg + (size_t)row * xg_ld + c, xg_lo, xv[0], xv[1], xv[2], xv[3]);
    float sq = (acc.x * acc.x + acc.y * acc.y) + (acc.z * acc.z + acc.w * acc.w);
    sq += __shfl_xor(sq, 1, 64);
    sq += __shfl_xor(sq, 2, 64);
    if ((threadIdx.x & 3) == 0) ss[(size_t)row * ss_stride + (c >> 4)] = sq;
  }
}

__global__ void moe_copy_choices_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int layers,
                                        int per_layer_src, int per_layer_dst) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= layers * per_layer_dst) return;
  dst[i] = src[(size_t)(i / per_layer_dst) * per_layer_src + i % per_layer_dst];
}

void launch_moe_route(hipStream_t st, const float* logits, int E, int top_k, const int32_t* m_count, int rows_cap,
                      int32_t* choice, float* route_w) {
  S2D2_LAUNCH(moe_route_kernel, dim3((rows_cap + 3) / 4), dim3(256), 0, st, logits, E, top_k, m_count, choice,
                     route_w);
}

void launch_moe_group(hipStream_t st, int E, int top_k, const int32_t* m_count, const int32_t* choice,
                      int32_t* sorted, int32_t* tile_expert, int32_t* tile_row0, int32_t* tile_rows, int32_t* n_tiles,
                      int tile_cap) {
  S2D2_LAUNCH(moe_group_kernel, dim3(1), dim3(1024), 0, st, E, top_k, m_count, choice, sorted,
                     tile_expert, tile_row0, tile_rows, n_tiles, tile_cap);
}

void launch_moe_combine(hipStream_t st, const float* y, int d, int top_k, const int32_t* m_count, int rows_cap,
                        float* h, void* xg, int xg_ld, int xg_lo, const float* gain_next, float* ss, int ss_stride) {
  S2D2_LAUNCH(moe_combine_kernel, dim3(rows_cap), dim3(256), 0, st, y, d, top_k, m_count, h, (bf16_t*)xg,
                     xg_ld, xg_lo, gain_next, ss, ss_stride);
}

void launch_moe_copy_choices(hipStream_t st, const int32_t* src, int32_t* dst, int layers, int per_layer_src,
                             int per_layer_dst) {
  const int n = layers * per_layer_dst;
  S2D2_LAUNCH(moe_copy_choices_kernel, dim3((n + 255) / 256), dim3(256), 0, st, src, dst, layers, per_layer_src,
                     per_layer_dst);
}

}  // namespace s2d2
