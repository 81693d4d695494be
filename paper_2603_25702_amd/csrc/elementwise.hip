// Row-wise kernels of the decoder forward: embedding gather, RMSNorm, RoPE + q/k/v split.
// All are HBM/L2-bound copies with a little arithmetic; one workgroup per window row.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

namespace s2d2 {

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T* __restrict__ embed, int d, Plan p,
                                                    float* __restrict__ h) {
  const int r = blockIdx.x;
  if (r >= p.counts[0]) return;
  const T* src = embed + (size_t)p.row_token[r] * d;
  float* dst = h + (size_t)r * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = to_f32(src[i]);
}

void launch_embed(hipStream_t st, int dtype, const void* embed, int d, const Plan& p, int rows_cap, float* h) {
  if (dtype == S2D2_BF16)
    S2D2_LAUNCH(embed_kernel<bf16_t>, dim3(rows_cap), dim3(256), 0, st, (const bf16_t*)embed, d, p, h);
  else
    S2D2_LAUNCH(embed_kernel<float>, dim3(rows_cap), dim3(256), 0, st, (const float*)embed, d, p, h);
}

__device__ __forceinline__ float block_sum_256(float v, float* red) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// out[r, :] = h[src, :] * rsqrt(mean(h[src, :]^2) + eps) * gain
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ h,
                                                      const float* __restrict__ gain, int d, float eps,
                                                      const int32_t* __restrict__ count,
                                                      const int32_t* __restrict__ gather, T* __restrict__ out) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  if (r >= *count) return;
  const float* x = h + (size_t)(gather ? gather[r] : r) * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) { const float v = x[i]; ss += v * v; }
  ss = block_sum_256(ss, red);
  const float rs = 1.0f / sqrtf(ss / (float)d + eps);
  T* o = out + (size_t)r * d;
  for (int i = threadIdx.x; i < d; i += 256) o[i] = from_f32<T>(x[i] * rs * gain[i]);
}

void launch_rmsnorm(hipStream_t st, int dtype, const float* h, const float* gain, int d, float eps,
                    const int32_t* count, const int32_t* gather, int rows_cap, void* out) {
  if (dtype == S2D2_BF16)
    S2D2_LAUNCH(rmsnorm_kernel<bf16_t>, dim3(rows_cap), dim3(256), 0, st, h, gain, d, eps, count, gather,
                       (bf16_t*)out);
  else
    S2D2_LAUNCH(rmsnorm_kernel<float>, dim3(rows_cap), dim3(256), 0, st, h, gain, d, eps, count, gather,
                       (float*)out);
}

// qkv fp32 [rows, (Hq + 2 Hkv) D] -> q [rows, Hq, D] (RoPE), k [rows, Hkv, D] (RoPE), v [rows, Hkv, D].
// Half-split pairing: element i rotates with element i + D/2 by pos * theta^(-2i/D).  The phase is
// computed in fp64 so that positions in the thousands keep full fp32 accuracy in sin / cos.
template <typename T>
__global__ __launch_bounds__(256) void rope_split_kernel(const float* __restrict__ qkv, Plan p, int Hq, int Hkv,
                                                         int D, float theta, T* __restrict__ q_out,
                                                         T* __restrict__ k_out, T* __restrict__ v_out,
                                                         T* __restrict__ vT_out, int wpad) {
  __shared__ float s_cos[128], s_sin[128];
  const int r = blockIdx.x;
  if (r >= p.counts[0]) return;
  const int half = D >> 1;
  const double pos = (double)p.row_pos[r];
  for (int i = threadIdx.x; i < half; i += 256) {
    const double inv = exp2(-2.0 * (double)i / (double)D * log2((double)theta));
    double s, c;
    sincos(pos * inv, &s, &c);
    s_cos[i] = (float)c;
    s_sin[i] = (float)s;
  }
  __syncthreads();
  const float* x = qkv + (size_t)r * (Hq + 2 * Hkv) * D;
  const int n_rot = (Hq + Hkv) * half;  // rotated pairs (q heads then k heads)
  for (int e = threadIdx.x; e < n_rot; e += 256) {
    const int hd = e / half, i = e % half;
    const float x1 = x[hd * D + i], x2 = x[hd * D + i + half];
    const float y1 = x1 * s_cos[i] - x2 * s_sin[i];
    const float y2 = x2 * s_cos[i] + x1 * s_sin[i];
    T* dst = hd < Hq ? q_out + ((size_t)r * Hq + hd) * D : k_out + ((size_t)r * Hkv + (hd - Hq)) * D;
    dst[i] = from_f32<T>(y1);
    dst[i + half] = from_f32<T>(y2);
  }
  const float* xv = x + (size_t)(Hq + Hkv) * D;
  T* vd = v_out + (size_t)r * Hkv * D;
  for (int e = threadIdx.x; e < Hkv * D; e += 256) vd[e] = from_f32<T>(xv[e]);
  if (vT_out) {  // key-minor copy of the window's V for the MFMA attention: [seq, Hkv, D, wpad]
    const int n = p.row_seq[r], t = r - p.seq_row0[n];
    T* vt = vT_out + (size_t)n * Hkv * D * wpad + t;
    for (int e = threadIdx.x; e < Hkv * D; e += 256) vt[(size_t)e * wpad] = from_f32<T>(xv[e]);
  }
}

void launch_rope_split(hipStream_t st, int dtype, const float* qkv, const Plan& p, int rows_cap, int Hq,
                       int Hkv, int D, float theta, void* q_out, void* k_out, void* v_out, void* vT_out, int wpad) {
  if (dtype == S2D2_BF16)
    S2D2_LAUNCH(rope_split_kernel<bf16_t>, dim3(rows_cap), dim3(256), 0, st, qkv, p, Hq, Hkv, D, theta,
                       (bf16_t*)q_out, (bf16_t*)k_out, (bf16_t*)v_out, (bf16_t*)vT_out, wpad);
  else
    S2D2_LAUNCH(rope_split_kernel<float>, dim3(rows_cap), dim3(256), 0, st, qkv, p, Hq, Hkv, D, theta,
                       (float*)q_out, (float*)k_out, (float*)v_out, (float*)vT_out, wpad);
}

}  // namespace s2d2
