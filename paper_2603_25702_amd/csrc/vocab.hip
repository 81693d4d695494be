// Vocabulary-wide kernels: SampleFromLogits / ScoreFromLogits statistics, the threshold set of
// Algorithm 2, and the accept scan + residual resampling of Algorithm 3.
//
// The statistics kernels stream each fp32 logit row exactly once with 16-byte coalesced loads
// (HBM-bound: rows * V * 4 bytes), keep an online (max, sum-exp, entropy numerator, arg-max,
// second max) per lane, and reduce with wavefront shuffles, then LDS, then a fixed-order merge
// over the row's chunks, so results do not depend on scheduling.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

#include <mutex>

namespace s2d2 {

static constexpr int VCHUNK = 4096;  // logits per workgroup: 256 lanes x 4 float4

int vocab_chunks(int V) { return (V + VCHUNK - 1) / VCHUNK; }

struct Stat {
  float m;    // max logit
  float z;    // sum exp(l - m)
  float e;    // sum exp(l - m) * (l - m)
  float m2;   // second largest logit (equals m if the max is attained twice)
  int arg;    // lowest index attaining m
};

__device__ __forceinline__ Stat stat_empty() { return Stat{-INFINITY, 0.f, 0.f, -INFINITY, 0x7fffffff}; }

__device__ __forceinline__ Stat stat_merge(const Stat& a, const Stat& b) {
  Stat r;
  r.m = fmaxf(a.m, b.m);
  r.arg = a.m > b.m ? a.arg : (b.m > a.m ? b.arg : min(a.arg, b.arg));
  r.m2 = fmaxf(fminf(a.m, b.m), fmaxf(a.m2, b.m2));
  const float da = a.m - r.m, db = b.m - r.m;  // <= 0, or NaN when both are -inf
  const float fa = a.z > 0.f ? __expf(da) : 0.f, fb = b.z > 0.f ? __expf(db) : 0.f;
  r.z = a.z * fa + b.z * fb;
  r.e = (a.z > 0.f ? fa * (a.e + da * a.z) : 0.f) + (b.z > 0.f ? fb * (b.e + db * b.z) : 0.f);
  return r;
}

__device__ __forceinline__ Stat stat_shfl_xor(const Stat& s, int off) {
  Stat r;
  r.m = __shfl_xor(s.m, off, 64);
  r.z = __shfl_xor(s.z, off, 64);
  r.e = __shfl_xor(s.e, off, 64);
  r.m2 = __shfl_xor(s.m2, off, 64);
  r.arg = __shfl_xor(s.arg, off, 64);
  return r;
}

// part[row][chunk][8] = {m, z, e, m2, arg}
// inv_t: 1 / temperature (1 in greedy mode: the multiplication is then exact); all statistics are those of
// softmax(logits * inv_t).
__global__ __launch_bounds__(256) void vocab_partial_kernel(const float* __restrict__ logits, int V,
                                                            const int32_t* __restrict__ count, int chunks,
                                                            float inv_t, float* __restrict__ part) {
  __shared__ Stat s_w[4];
  const int row = blockIdx.y, chunk = blockIdx.x;
  if (row >= *count) return;
  const float* x = logits + (size_t)row * V;
  const int base = chunk * VCHUNK;
  const int tid = threadIdx.x;
  float v[16];
  int idx0[4];
  const bool vec_ok = (V & 3) == 0;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int i = base + t * 1024 + tid * 4;
    idx0[t] = i;
    if (vec_ok && i + 3 < V) {
      const float4 f = *(const float4*)(x + i);
      v[4 * t] = f.x * inv_t; v[4 * t + 1] = f.y * inv_t; v[4 * t + 2] = f.z * inv_t; v[4 * t + 3] = f.w * inv_t;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[4 * t + e] = (i + e < V) ? x[i + e] * inv_t : -INFINITY;
    }
  }
  Stat s = stat_empty();
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    const float l = v[t];
    const int i = idx0[t >> 2] + (t & 3);
    if (l > s.m) { s.m2 = s.m; s.m = l; s.arg = i; }
    else if (l > s.m2) s.m2 = l;
  }
  if (s.m > -INFINITY) {
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const float d = v[t] - s.m;
      const float ex = __expf(d);          // exp(-inf) = 0 for padded slots
      s.z += ex;
      s.e += ex > 0.f ? ex * d : 0.f;
    }
  }
  for (int off = 1; off < 64; off <<= 1) s = stat_merge(s, stat_shfl_xor(s, off));
  if ((tid & 63) == 0) s_w[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    Stat r = stat_merge(stat_merge(s_w[0], s_w[1]), stat_merge(s_w[2], s_w[3]));
    float* o = part + ((size_t)row * chunks + chunk) * 8;
    o[0] = r.m; o[1] = r.z; o[2] = r.e; o[3] = r.m2; o[4] = __int_as_float(r.arg);
  }
}

// Chunk partials of one row, merged by one wavefront: lane c takes chunks c, c + 64, ..., then a butterfly over the
// lanes (a fixed order; stat_merge is symmetric, ties go to the lower index).  One thread walking the 38 chunks of a
// 152k vocabulary one after the other took 8-10 us per launch.  Lane 0's result is the one that is used.
__device__ __forceinline__ Stat merge_chunks(const float* part, int row, int chunks) {
  Stat r = stat_empty();
  for (int c = threadIdx.x & 63; c < chunks; c += 64) {
    const float* o = part + ((size_t)row * chunks + c) * 8;
    Stat s{o[0], o[1], o[2], o[3], __float_as_int(o[4])};
    r = stat_merge(r, s);
  }
  for (int off = 1; off < 64; off <<= 1) r = stat_merge(r, stat_shfl_xor(r, off));
  return r;
}

// SampleFromLogits (greedy): x_hat = arg-max, p = softmax probability of it, plus lse, margin, H/ln V.
__global__ void vocab_draft_final_kernel(const float* __restrict__ part, int chunks, int V,
                                         const int32_t* __restrict__ count,
                                         const int32_t* __restrict__ logit_seq,
                                         const int32_t* __restrict__ logit_idx, int B,
                                         int32_t* __restrict__ xhat, float* __restrict__ p,
                                         float* __restrict__ lse, float* __restrict__ margin,
                                         float* __restrict__ entropy_n) {
  const int row = blockIdx.x;   // one wavefront per logit row
  if (row >= *count) return;
  const Stat s = merge_chunks(part, row, chunks);
  if (threadIdx.x != 0) return;
  const int o = logit_seq ? logit_seq[row] * B + logit_idx[row] : row;
  const float inv = 1.0f / s.z;
  xhat[o] = s.arg < V ? s.arg : 0;   // no comparable logit in the row (all NaN): the first index, as an arg-max over NaNs gives
  p[o] = inv;
  lse[o] = s.m + logf(s.z);
  margin[o] = inv - expf(s.m2 - s.m) * inv;
  entropy_n[o] = fmaxf(0.f, logf(s.z) - s.e * inv) / logf((float)V);
}

// ScoreFromLogits: q = softmax(logits_ver)[token], lse.
__global__ void vocab_score_final_kernel(const float* __restrict__ part, int chunks, int V,
                                         const float* __restrict__ logits, const int32_t* __restrict__ count,
                                         const int32_t* __restrict__ logit_seq,
                                         const int32_t* __restrict__ logit_idx, int B,
                                         const int32_t* __restrict__ token, float inv_t, float* __restrict__ q,
                                         float* __restrict__ lse) {
  const int row = blockIdx.x;   // one wavefront per logit row
  if (row >= *count) return;
  const Stat s = merge_chunks(part, row, chunks);
  if (threadIdx.x != 0) return;
  const int o = logit_seq ? logit_seq[row] * B + logit_idx[row] : row;
  const float l = s.m + logf(s.z);
  const int tok = token[o];
  lse[o] = l;
  q[o] = (tok >= 0 && tok < V) ? expf(logits[(size_t)row * V + tok] * inv_t - l) : 0.f;
}

__global__ void vocab_sample_kernel(const float* __restrict__ logits, int V, const int32_t* __restrict__ count,
                                    const int32_t* __restrict__ logit_seq, const int32_t* __restrict__ logit_idx, int B,
                                    uint64_t seed, uint32_t step, const uint32_t* __restrict__ step_dev, float inv_t,
                                    const float* __restrict__ lse, int32_t* __restrict__ xhat, float* __restrict__ p);

void launch_vocab_draft(hipStream_t st, const float* logits, int V, const int32_t* count, int rows_cap,
                        const VocabWs& ws, const int32_t* logit_seq, const int32_t* logit_idx, int B,
                        int32_t* xhat, float* p, float* lse, float* margin, float* entropy_n, const VocabSample& sm) {
  const float inv_t = sm.sample ? 1.0f / sm.temperature : 1.0f;
  S2D2_LAUNCH(vocab_partial_kernel, dim3(ws.chunks, rows_cap), dim3(256), 0, st, logits, V, count,
                     ws.chunks, inv_t, ws.part);
  S2D2_LAUNCH(vocab_draft_final_kernel, dim3(rows_cap), dim3(64), 0, st, ws.part, ws.chunks, V,
                     count, logit_seq, logit_idx, B, xhat, p, lse, margin, entropy_n);
  if (sm.sample)
    S2D2_LAUNCH(vocab_sample_kernel, dim3(rows_cap), dim3(256), 0, st, logits, V, count, logit_seq, logit_idx, B,
                sm.seed, sm.step, sm.step_dev, inv_t, lse, xhat, p);
}

void launch_vocab_score(hipStream_t st, const float* logits, int V, const int32_t* count, int rows_cap,
                        const VocabWs& ws, const int32_t* logit_seq, const int32_t* logit_idx, int B,
                        const int32_t* token, float* q, float* lse, float inv_t) {
  S2D2_LAUNCH(vocab_partial_kernel, dim3(ws.chunks, rows_cap), dim3(256), 0, st, logits, V, count,
                     ws.chunks, inv_t, ws.part);
  S2D2_LAUNCH(vocab_score_final_kernel, dim3(rows_cap), dim3(64), 0, st, ws.part, ws.chunks, V,
                     logits, count, logit_seq, logit_idx, B, token, inv_t, q, lse);
}

// Per sequence: defaults for committed positions, threshold set S = {i in M: p_i > tau} U {argmax p}.
__global__ void draft_finish_kernel(int N, int B, int mask_id, float tau, const int32_t* __restrict__ block,
                                    int32_t* __restrict__ xhat, float* __restrict__ p, float* __restrict__ lse,
                                    float* __restrict__ margin, float* __restrict__ entropy_n,
                                    uint64_t* __restrict__ unmask, int32_t* __restrict__ n_hi) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  uint64_t bits = 0;
  int hi = 0, best = -1;
  float best_p = -1.f;
  for (int i = 0; i < B; ++i) {
    const int o = n * B + i;
    if (block[o] == mask_id) {
      const float pi = p[o];
      if (pi > tau) { bits |= 1ull << i; ++hi; }
      if (pi > best_p) { best_p = pi; best = i; }   // strict: lowest index wins ties
    } else {
      xhat[o] = -1; p[o] = 0.f; lse[o] = 0.f; margin[o] = 0.f; entropy_n[o] = 0.f;
    }
  }
  if (best >= 0) bits |= 1ull << best;
  unmask[n] = bits;
  n_hi[n] = hi;
}

void launch_draft_finish(hipStream_t st, int N, int B, int mask_id, float tau, const int32_t* block,
                         int32_t* xhat, float* p, float* lse, float* margin, float* entropy_n,
                         uint64_t* unmask, int32_t* n_hi) {
  S2D2_LAUNCH(draft_finish_kernel, dim3((N + 63) / 64), dim3(64), 0, st, N, B, mask_id, tau, block, xhat, p,
                     lse, margin, entropy_n, unmask, n_hi);
}

// ---------------------------------------------------------------------------------------------
// Counter-based uniforms: Philox-4x32 with 10 rounds (Salmon et al., SC'11), written from the
// published round function.  key = seed, counter = (step, sequence, block index, stream).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t philox_first_word(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                      uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

__device__ __forceinline__ float uniform01(uint64_t seed, uint32_t step, uint32_t seq, uint32_t idx, uint32_t stream) {
  const uint32_t w = philox_first_word(step, seq, idx, stream, (uint32_t)seed, (uint32_t)(seed >> 32));
  return ((float)(w >> 9) + 0.5f) * (1.0f / 8388608.0f);  // odd multiple of 2^-24: exact
}

// Scan of one non-negative float per thread over a 256-thread block with a fixed tree.
// Returns the inclusive prefix; *excl is the inclusive prefix of the previous thread (0 for
// thread 0), so the intervals [excl, incl) of consecutive threads tile [0, total) exactly;
// *total is the inclusive prefix of the last thread.  s_w needs 4 floats.  Threads past the first 256 (a wider
// workgroup) must pass 0 and get an empty interval at the total.
__device__ __forceinline__ float block_scan_256(float v, float* s_w, float* excl, float* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int off = 1; off < 64; off <<= 1) {
    const float t = __shfl_up(v, off, 64);
    if (lane >= off) v += t;
  }
  __syncthreads();
  if (lane == 63 && w < 4) s_w[w] = v;
  __syncthreads();
  float pre = 0.f;
  for (int i = 0; i < min(w, 4); ++i) pre += s_w[i];
  const float incl = v + pre;
  const float prev = __shfl_up(incl, 1, 64);
  *excl = lane == 0 ? pre : prev;
  *total = s_w[3] + ((s_w[0] + s_w[1]) + s_w[2]);
  return incl;
}

static constexpr int RTILE = 256;     // residual tile: one wavefront x float4
static constexpr int RMAX_TILES = 8192;

// Inverse CDF over V non-negative weights in ascending index order, by a workgroup of 256 threads or more (the tile sums use all of them):
// returns (in the lanes of wavefront 0; -1 elsewhere) the smallest index whose inclusive prefix sum exceeds
// u * total, or -1 if the weights have no mass.  w4(i0, r) yields the weights of indices i0 .. i0+3 (zeros
// past V).  Two levels with a fixed summation order: tile sums (256 indices per tile: one wavefront x 4),
// a scan of the tile sums, then a walk of the selected tile; rounding at either level falls back to the
// nearest index that has mass.  s_tile needs RMAX_TILES floats, s_w four.
// First level: the sums of tiles [tb, te) go to dst[tile] (LDS, or global memory with device-coherent stores when
// several workgroups share the tiles of one row).  Eight tiles of a wavefront at a time: their loads are all issued
// before the first reduction (one tile per iteration made the pass a chain of ~150 memory round trips per
// wavefront).  A tile's sum does not depend on which wavefront or workgroup forms it.
template <bool COH, typename F>
__device__ __forceinline__ void inverse_cdf_tile_sums(const F& w4, int tb, int te, float* dst) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  constexpr int TU = 8;
  const int nw = blockDim.x >> 6;   // every wavefront of the workgroup takes part in this pass; the scan uses 256 threads
  for (int t0 = tb + w * TU; t0 < te; t0 += nw * TU) {
    float r4[TU][4];
#pragma unroll
    for (int u_ = 0; u_ < TU; ++u_) w4((t0 + u_) * RTILE + lane * 4, r4[u_]);   // indices at or past V give zeros
#pragma unroll
    for (int u_ = 0; u_ < TU; ++u_) {
      float r = ((r4[u_][0] + r4[u_][1]) + r4[u_][2]) + r4[u_][3];
      for (int off = 32; off > 0; off >>= 1) r += __shfl_xor(r, off, 64);
      if (lane == 0 && t0 + u_ < te) {
        if (COH) st4f_coh(&dst[t0 + u_], r); else dst[t0 + u_] = r;
      }
    }
  }
}

// Second and third level, from the tile sums in s_tile (written by this workgroup's threads before the call).
template <typename F>
__device__ __forceinline__ int inverse_cdf_finish(const F& w4, int V, float u, float* s_tile, float* s_w,
                                                  int* s_tile_sel, float* s_before) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int tiles = (V + RTILE - 1) / RTILE;
  __syncthreads();
  // scan tile sums: thread t owns tiles [t*per, (t+1)*per)
  const int per = (tiles + 255) / 256;   // (threads past the first 256 own no tiles)
  float mine = 0.f;
  for (int t = tid * per; t < min(tiles, (tid + 1) * per); ++t) mine += s_tile[t];
  float total, excl;
  const float incl = block_scan_256(mine, s_w, &excl, &total);
  const float target = u * total;
  if (tid == 0) { *s_tile_sel = -1; *s_before = 0.f; }
  __syncthreads();
  if (excl <= target && target < incl) {  // exactly one thread: the intervals tile [0, total)
    float run = excl, before = excl;
    int sel = -1, last = -1;
    for (int t = tid * per; t < min(tiles, (tid + 1) * per); ++t) {
      const float ts = s_tile[t];
      if (ts > 0.f) { last = t; before = run; }
      if (ts > 0.f && run + ts > target) { sel = t; break; }
      run += ts;
    }
    if (sel < 0) sel = last;          // rounding: take the thread's last tile that has mass
    *s_tile_sel = sel;
    *s_before = before;
  }
  __syncthreads();
  int sel = *s_tile_sel;
  int token = -1;
  if (total > 0.f && sel < 0) {  // target landed at or beyond the total by rounding: last tile with mass
    if (tid == 0) {
      for (int t = tiles - 1; t >= 0; --t)
        if (s_tile[t] > 0.f) { *s_tile_sel = t; break; }
      float run = 0.f;
      for (int t = 0; t < *s_tile_sel; ++t) run += s_tile[t];
      *s_before = run;
    }
    __syncthreads();
    sel = *s_tile_sel;
  }
  if (total > 0.f && sel >= 0 && w == 0) {  // wave 0 walks the selected tile in index order
    const int i0 = sel * RTILE + lane * 4;
    float r4[4];
    w4(i0, r4);
    const float ls = ((r4[0] + r4[1]) + r4[2]) + r4[3];
    float inc = ls;
    for (int off = 1; off < 64; off <<= 1) {
      const float t = __shfl_up(inc, off, 64);
      if (lane >= off) inc += t;
    }
    float run = *s_before + (inc - ls);
    int cand = 0x7fffffff, last_pos = -1;
    for (int e = 0; e < 4; ++e) {
      if (r4[e] > 0.f) last_pos = i0 + e;
      run += r4[e];
      if (cand == 0x7fffffff && r4[e] > 0.f && run > target) cand = i0 + e;
    }
    for (int off = 32; off > 0; off >>= 1) {
      cand = min(cand, __shfl_xor(cand, off, 64));
      last_pos = max(last_pos, __shfl_xor(last_pos, off, 64));
    }
    token = cand != 0x7fffffff ? cand : last_pos;
  }
  return token;
}

template <typename F>
__device__ __forceinline__ int inverse_cdf_block(const F& w4, int V, float u, float* s_tile, float* s_w,
                                                 int* s_tile_sel, float* s_before) {
  inverse_cdf_tile_sums<false>(w4, 0, (V + RTILE - 1) / RTILE, s_tile);
  return inverse_cdf_finish(w4, V, u, s_tile, s_w, s_tile_sel, s_before);
}

// SampleFromLogits in sampling mode: x_hat ~ softmax(logits / T) by inverse CDF in ascending vocabulary order with
// the uniform of stream 2 at (step, sequence, block index); p = that token's probability.  One workgroup per
// logit row; runs after the statistics kernels (reads lse, overwrites the arg-max proposal and its probability).
__global__ __launch_bounds__(256) void vocab_sample_kernel(
    const float* __restrict__ logits, int V, const int32_t* __restrict__ count, const int32_t* __restrict__ logit_seq,
    const int32_t* __restrict__ logit_idx, int B, uint64_t seed, uint32_t step, const uint32_t* __restrict__ step_dev,
    float inv_t, const float* __restrict__ lse, int32_t* __restrict__ xhat, float* __restrict__ p) {
  __shared__ float s_tile[RMAX_TILES];
  __shared__ float s_w[4];
  __shared__ int s_tile_sel;
  __shared__ float s_before;
  const int row = blockIdx.x;
  if (row >= *count) return;
  const int n = logit_seq ? logit_seq[row] : row, idx = logit_idx ? logit_idx[row] : 0;
  const int o = logit_seq ? n * B + idx : row;
  const float* x = logits + (size_t)row * V;
  const float z = lse[o];
  const uint32_t stp = step + (step_dev ? *step_dev : 0u);
  const float u = uniform01(seed, stp, (uint32_t)n, (uint32_t)idx, 2u);
  auto prob4 = [&](int i0, float (&r)[4]) {
    if ((V & 3) == 0) {   // unconditional load (clamped index) so that the loads of several tiles can be in flight
      const bool ok = i0 < V;
      const float4 a = *(const float4*)(x + (ok ? i0 : 0));
      r[0] = ok ? __expf(a.x * inv_t - z) : 0.f; r[1] = ok ? __expf(a.y * inv_t - z) : 0.f;
      r[2] = ok ? __expf(a.z * inv_t - z) : 0.f; r[3] = ok ? __expf(a.w * inv_t - z) : 0.f;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] = (i0 + e < V) ? __expf(x[i0 + e] * inv_t - z) : 0.f;
    }
  };
  const int token = inverse_cdf_block(prob4, V, u, s_tile, s_w, &s_tile_sel, &s_before);
  if (threadIdx.x == 0 && token >= 0) {   // (no mass cannot happen for a softmax; the arg-max proposal would stay)
    xhat[o] = token;
    p[o] = expf(x[token] * inv_t - z);
  }
}

// gridDim.y workgroups per sequence: accept scan over C_t (thread 0 of each, the same result in all), then, if a
// drafted token failed, a draw from the residual (P_ver - P_draft)_+ by inverse CDF in ascending vocabulary order.
// With several workgroups each forms the tile sums of its share of the vocabulary (one sequence alone would stream
// its two logit rows through a single compute unit), leaves them in tile_scratch[sequence][tile] and counts its
// arrival; the last one to arrive finishes the draw and re-arms the counter.  Workgroup 0 writes everything that
// does not depend on the draw.  The result does not depend on gridDim.y.
__global__ __launch_bounds__(1024) void accept_kernel(
    int B, int V, uint64_t seed, uint32_t step, const uint32_t* __restrict__ step_dev, float gamma, int resample,
    float inv_t, const int32_t* __restrict__ span_start, const int32_t* __restrict__ span_len,
    const float* __restrict__ logits_d, const int32_t* __restrict__ row_of_d,
    const float* __restrict__ logits_v, const int32_t* __restrict__ row_of_v,
    const int32_t* __restrict__ xhat, const float* __restrict__ p, const float* __restrict__ lse_d,
    const float* __restrict__ q, const float* __restrict__ lse_v, int32_t* __restrict__ block,
    int32_t* __restrict__ n_accept, int32_t* __restrict__ n_commit, int32_t* __restrict__ resampled,
    float* __restrict__ u_used, const int32_t* __restrict__ active, float* __restrict__ tile_scratch,
    int32_t* __restrict__ arrivals) {
  __shared__ float s_tile[RMAX_TILES];
  __shared__ float s_w[4];
  __shared__ int s_nacc, s_last;
  __shared__ int s_tile_sel;
  __shared__ float s_before;
  const int n = blockIdx.x, tid = threadIdx.x, g = blockIdx.y, G = gridDim.y;
  const int j = span_start[n], L = (active && active[n] == 0) ? 0 : span_len[n];   // not routed to the verifier: nothing to scan
  const uint32_t stp = step + (step_dev ? *step_dev : 0u);
  if (g == 0)
    for (int i = tid; i < B; i += blockDim.x) u_used[(size_t)n * B + i] = 0.f;
  __syncthreads();
  if (tid == 0) {
    int acc = 0;
    for (; acc < L; ++acc) {
      const int o = n * B + j + acc;
      const float u = uniform01(seed, stp, (uint32_t)n, (uint32_t)(j + acc), 0u);
      if (g == 0) u_used[o] = u;
      const float pi = p[o], qi = q[o];
      const bool ok = gamma == 1.0f ? (u * pi < qi) : (u < fminf(1.0f, powf(qi / pi, gamma)));
      if (!ok) break;
    }
    s_nacc = acc;
  }
  __syncthreads();
  const int acc = s_nacc;
  if (g == 0)
    for (int i = tid; i < acc; i += blockDim.x) block[n * B + j + i] = xhat[n * B + j + i];
  if (acc >= L || !resample) {
    if (g == 0 && tid == 0) { n_accept[n] = acc; n_commit[n] = acc; resampled[n] = -1; }
    return;
  }
  // ---- residual at block index i: r(v) = max(0, Q(v) - P(v)), both at the sampling temperature ----
  const int o = n * B + j + acc;
  const float* ld = logits_d + (size_t)row_of_d[o] * V;
  const float* lv = logits_v + (size_t)row_of_v[o] * V;
  const float zd = lse_d[o], zv = lse_v[o];
  const float u2 = uniform01(seed, stp, (uint32_t)n, (uint32_t)(j + acc), 1u);
  auto residual4 = [&](int i0, float (&r)[4]) {
    if ((V & 3) == 0) {   // unconditional loads (clamped index) so that the loads of several tiles can be in flight
      const bool ok = i0 < V;
      const int ic = ok ? i0 : 0;
      const float4 a = *(const float4*)(ld + ic), b = *(const float4*)(lv + ic);
      r[0] = ok ? fmaxf(0.f, __expf(b.x * inv_t - zv) - __expf(a.x * inv_t - zd)) : 0.f;
      r[1] = ok ? fmaxf(0.f, __expf(b.y * inv_t - zv) - __expf(a.y * inv_t - zd)) : 0.f;
      r[2] = ok ? fmaxf(0.f, __expf(b.z * inv_t - zv) - __expf(a.z * inv_t - zd)) : 0.f;
      r[3] = ok ? fmaxf(0.f, __expf(b.w * inv_t - zv) - __expf(a.w * inv_t - zd)) : 0.f;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        r[e] = (i0 + e < V) ? fmaxf(0.f, __expf(lv[i0 + e] * inv_t - zv) - __expf(ld[i0 + e] * inv_t - zd)) : 0.f;
    }
  };
  int token;
  if (G == 1) {
    token = inverse_cdf_block(residual4, V, u2, s_tile, s_w, &s_tile_sel, &s_before);
  } else {
    const int tiles = (V + RTILE - 1) / RTILE, share = (tiles + G - 1) / G;
    float* mine = tile_scratch + (size_t)n * tiles;
    inverse_cdf_tile_sums<true>(residual4, min(tiles, g * share), min(tiles, (g + 1) * share), mine);
    __builtin_amdgcn_s_waitcnt(0);   // the write-through stores have completed before the arrival is counted
    __syncthreads();
    if (tid == 0) {
      const int prev = __hip_atomic_fetch_add(&arrivals[n], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = prev == G - 1;
      if (prev == G - 1) __hip_atomic_store(&arrivals[n], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!s_last) return;
    for (int t = tid; t < tiles; t += blockDim.x) s_tile[t] = ld4f_coh(&mine[t]);
    token = inverse_cdf_finish(residual4, V, u2, s_tile, s_w, &s_tile_sel, &s_before);
  }
  if (tid == 0) {
    if (token < 0) token = xhat[o];  // residual without mass in fp32 (p and q equal to rounding): keep the draft
    block[o] = token;
    n_accept[n] = acc;
    n_commit[n] = acc + 1;
    resampled[n] = token;
  }
}

void launch_accept(hipStream_t st, int N, int B, int V, uint64_t seed, uint32_t step, const uint32_t* step_dev,
                   float gamma, int resample, float inv_t, const int32_t* span_start, const int32_t* span_len,
                   const float* logits_d, const int32_t* row_of_d, const float* logits_v,
                   const int32_t* row_of_v, const int32_t* xhat, const float* p, const float* lse_d,
                   const float* q, const float* lse_v, int32_t* block, int32_t* n_accept, int32_t* n_commit,
                   int32_t* resampled, float* u_used, const int32_t* active, float* tile_scratch, int32_t* arrivals) {
  // few sequences: up to 8 workgroups share the vocabulary of each (a share is then one round of the tile pass for
  // vocabularies of up to 2^18 entries)
  const int G = tile_scratch && arrivals ? std::max(1, std::min(8, 128 / N)) : 1;
  S2D2_LAUNCH(accept_kernel, dim3(N, G), dim3(1024), 0, st, B, V, seed, step, step_dev, gamma, resample, inv_t,
                     span_start, span_len, logits_d, row_of_d, logits_v, row_of_v, xhat, p, lse_d, q, lse_v, block,
                     n_accept, n_commit, resampled, u_used, active, tile_scratch, arrivals);
}

size_t accept_tile_floats(int max_batch, int V) { return (size_t)max_batch * ((V + RTILE - 1) / RTILE); }

// ---------------------------------------------------------------------------------------------
// Scratch of the accept step for callers that cannot allocate (s2d2_accept_static): the residual tile sums that
// the workgroups of a sequence hand to each other, and their arrival counters, live in a file-scope device array
// instead of the caller's workspace.  Every GPU holds its own copy of the array at its own address; the address
// is looked up once per device and only that pointer is ever passed to a kernel.
// ---------------------------------------------------------------------------------------------
static constexpr size_t STATIC_TILE_FLOATS = (size_t)ACCEPT_STATIC_MAX_BATCH * (ACCEPT_STATIC_MAX_VOCAB / RTILE);
static constexpr size_t STATIC_SCRATCH_BYTES = STATIC_TILE_FLOATS * sizeof(float) + ACCEPT_STATIC_MAX_BATCH * sizeof(int32_t);
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];   // 512.5 KB per GPU, held until the process ends

static constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[STATIC_MAX_DEVICES];   // device address of `scratch` on each GPU, once looked up

int accept_static_scratch(float** tiles, int32_t** arrivals) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) { (void)hipGetLastError(); return -1; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return -1; }
    g_scratch_ptr[dev] = ptr;
  }
  if (tiles) *tiles = (float*)g_scratch_ptr[dev];
  if (arrivals) *arrivals = (int32_t*)((unsigned char*)g_scratch_ptr[dev] + STATIC_TILE_FLOATS * sizeof(float));
  return 0;
}

}  // namespace s2d2
