// Y[m, n] = sum_k X[m, k] * W[n, k] on MFMA, fp32 accumulation.
//
// Weight-streaming kernel for the decode regime (a handful of window rows against a large
// weight matrix): the arithmetic intensity is ~M flop per weight byte, so the kernel is bound by
// reading W once from HBM.  One workgroup owns 16 output features and 16 rows; its four
// wavefronts split K and each lane streams 16-byte pieces of "its" weight row straight from
// global memory into the MFMA A operand (no LDS on the weight path), the rows of X (tiny,
// L2-resident) are the B operand.  Partial sums of the four waves are combined through LDS in
// a fixed order, so results are deterministic.  Larger M is covered by more row tiles.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

namespace s2d2 {

template <typename T> struct Mma;

template <> struct Mma<bf16_t> {
  static constexpr int KV = 8;  // elements per 16-byte fragment
  __device__ static __forceinline__ f32x4_t run(const uint4& a, const uint4& b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};

template <> struct Mma<float> {
  static constexpr int KV = 4;
  __device__ static __forceinline__ f32x4_t run(const uint4& a, const uint4& b, f32x4_t c) {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    return c;
  }
};

template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_rows16_kernel(const T* __restrict__ X, int ldx,
                                                          const T* __restrict__ W, int K, int N,
                                                          const int32_t* __restrict__ m_count,
                                                          void* __restrict__ out, int ldo) {
  constexpr int KV = Mma<T>::KV;
  constexpr int KSTEP = 4 * KV;      // k covered by one fragment load of the whole wave
  constexpr int U = 4;               // fragment loads in flight per operand
  constexpr int KC = U * KSTEP;
  constexpr int NACC = EPI == EPI_SWIGLU ? 2 : 1;
  __shared__ float red[4][NACC][256];

  const int M = *m_count;
  const int m0 = blockIdx.y * 16;
  if (m0 >= M) return;
  const int n0 = blockIdx.x * 16;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, f = lane & 15;

  const int wn = min(n0 + f, N - 1);
  const bool row_ok = (m0 + f) < M;
  const T* wp = W + (size_t)wn * K + g * KV;
  const T* wp2 = wp + (size_t)N * K;  // up projection (SwiGLU only)
  const T* xp = X + (size_t)(row_ok ? m0 + f : m0) * ldx + g * KV;

  f32x4_t acc[NACC];
  for (int a = 0; a < NACC; ++a) acc[a] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const uint4 zero = make_uint4(0, 0, 0, 0);

  for (int k0 = wave * KC; k0 < K; k0 += 4 * KC) {
    uint4 wa[U], wb[U], xb[U];
#pragma unroll
    for (int t = 0; t < U; ++t) {
      const int k = k0 + t * KSTEP;
      const bool ok = k < K;
      wa[t] = ok ? *(const uint4*)(wp + k) : zero;
      if (EPI == EPI_SWIGLU) wb[t] = ok ? *(const uint4*)(wp2 + k) : zero;
      xb[t] = (ok && row_ok) ? *(const uint4*)(xp + k) : zero;
    }
#pragma unroll
    for (int t = 0; t < U; ++t) {
      acc[0] = Mma<T>::run(wa[t], xb[t], acc[0]);
      if (EPI == EPI_SWIGLU) acc[NACC - 1] = Mma<T>::run(wb[t], xb[t], acc[NACC - 1]);
    }
  }
  // acc[a][i] = Y[m0 + f][n0 + 4 g + i]
  for (int a = 0; a < NACC; ++a)
    for (int i = 0; i < 4; ++i) red[wave][a][i * 64 + lane] = acc[a][i];
  __syncthreads();
  const int row = threadIdx.x >> 4, fe = threadIdx.x & 15;
  const int src = (fe & 3) * 64 + (fe >> 2) * 16 + row;
  float v[NACC];
  for (int a = 0; a < NACC; ++a) v[a] = (red[0][a][src] + red[1][a][src]) + (red[2][a][src] + red[3][a][src]);
  const int m = m0 + row, n = n0 + fe;
  if (m >= M || n >= N) return;
  if (EPI == EPI_STORE_F32) {
    ((float*)out)[(size_t)m * ldo + n] = v[0];
  } else if (EPI == EPI_ADD_F32) {
    ((float*)out)[(size_t)m * ldo + n] += v[0];
  } else {
    const float gate = v[0], up = v[NACC - 1];
    ((T*)out)[(size_t)m * ldo + n] = from_f32<T>(gate / (1.0f + __expf(-gate)) * up);
  }
}

template <typename T>
static void launch_t(hipStream_t st, GemmEpilogue epi, const T* X, int ldx, const T* W, int K, int N,
                     const int32_t* m_count, int m_cap, void* out, int ldo) {
  dim3 grid((N + 15) / 16, (m_cap + 15) / 16), block(256);
  switch (epi) {
    case EPI_STORE_F32:
      S2D2_LAUNCH((gemm_rows16_kernel<T, EPI_STORE_F32>), grid, block, 0, st, X, ldx, W, K, N, m_count, out, ldo);
      break;
    case EPI_ADD_F32:
      S2D2_LAUNCH((gemm_rows16_kernel<T, EPI_ADD_F32>), grid, block, 0, st, X, ldx, W, K, N, m_count, out, ldo);
      break;
    case EPI_SWIGLU:
      S2D2_LAUNCH((gemm_rows16_kernel<T, EPI_SWIGLU>), grid, block, 0, st, X, ldx, W, K, N, m_count, out, ldo);
      break;
  }
}

void launch_gemm(hipStream_t st, int dtype, GemmEpilogue epi, const void* X, int ldx, const void* W, int K,
                 int N, const int32_t* m_count, int m_cap, void* out, int ldo) {
  if (dtype == S2D2_BF16)
    launch_t<bf16_t>(st, epi, (const bf16_t*)X, ldx, (const bf16_t*)W, K, N, m_count, m_cap, out, ldo);
  else
    launch_t<float>(st, epi, (const float*)X, ldx, (const float*)W, K, N, m_count, m_cap, out, ldo);
}

}  // namespace s2d2
