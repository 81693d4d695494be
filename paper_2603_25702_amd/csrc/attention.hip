// Attention of one window row over the paged prefix cache plus the visible in-window keys.
//
// attn_generic_kernel: plain fp32 arithmetic, one workgroup per (window row, query head).  It is
// the reference-quality path (used for fp32 models and as the cross-check of the MFMA kernel):
// scores of all keys go to LDS, a block-wide softmax follows, then P*V with the head dimension
// across lanes.  Visibility inside the window follows the plan (Eq. 3 / Eq. 4): window row w is
// visible to row r iff row_lo[r] <= w < row_hi[r] or w == r; every cached position is visible.
#include "s2d2_internal.h"
#include "../../include/s2d2.h"
#include "attention_flash.h"

namespace s2d2 {

__device__ __forceinline__ float wave_max(float v) {
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_generic_kernel(
    const T* __restrict__ q, const T* __restrict__ k_win, const T* __restrict__ v_win,
    const T* __restrict__ k_pages, const T* __restrict__ v_pages, KvGeom g, Plan p, int Hq,
    T* __restrict__ o, float scale, int o_f16) {
  extern __shared__ float smem[];
  const int r = blockIdx.x, hq = blockIdx.y;
  if (r >= p.counts[0]) return;
  const int D = g.head_dim, Hkv = g.n_kv_heads, ps = g.page_size;
  const int kvh = hq / (Hq / Hkv);
  const int n = p.row_seq[r];
  const int S = max(0, min(g.seq_len[n], g.max_pages_per_seq * ps));
  const int row0 = p.seq_row0[n], nw = p.seq_rows[n];
  const int lo = p.row_lo[r], hi = p.row_hi[r];
  const int total = S + nw;
  float* s_q = smem;            // [D]
  float* s_red = smem + D;      // [256 + 8]
  float* s_sc = s_red + 264;    // [total]
  const int tid = threadIdx.x;

  for (int d = tid; d < D; d += 256) s_q[d] = to_f32(q[((size_t)r * Hq + hq) * D + d]) * scale;
  __syncthreads();

  const int32_t* pt = g.page_table + (size_t)n * g.max_pages_per_seq;
  float lmax = -INFINITY;
  for (int s = tid; s < total; s += 256) {
    const T* kp;
    bool vis = true;
    if (s < S) {
      const int page = min(max(pt[s / ps], 0), g.n_pages - 1);
      kp = k_pages + (((size_t)page * Hkv + kvh) * ps + (s % ps)) * D;
    } else {
      const int w = row0 + (s - S);
      vis = (w >= lo && w < hi) || w == r;
      kp = k_win + ((size_t)w * Hkv + kvh) * D;
    }
    float dot = -INFINITY;
    if (vis) {
      dot = 0.f;
      for (int d = 0; d < D; ++d) dot += s_q[d] * to_f32(kp[d]);
    }
    s_sc[s] = dot;
    lmax = fmaxf(lmax, dot);
  }
  lmax = wave_max(lmax);
  if ((tid & 63) == 0) s_red[tid >> 6] = lmax;
  __syncthreads();
  const float m = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  __syncthreads();
  float lsum = 0.f;
  for (int s = tid; s < total; s += 256) {
    const float e = __expf(s_sc[s] - m);   // exp(-inf) = 0 for invisible keys
    s_sc[s] = e;
    lsum += e;
  }
  lsum = wave_sum(lsum);
  if ((tid & 63) == 0) s_red[tid >> 6] = lsum;
  __syncthreads();
  const float denom = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
  __syncthreads();

  const int nslice = 256 / D, d = tid % D, sl = tid / D;
  float acc = 0.f;
  if (sl < nslice) {
    for (int s = sl; s < total; s += nslice) {
      const float pw = s_sc[s];
      if (pw == 0.f) continue;
      const T* vp;
      if (s < S) {
        const int page = min(max(pt[s / ps], 0), g.n_pages - 1);
        vp = v_pages + (((size_t)page * Hkv + kvh) * D + d) * ps + (s % ps);   // cache V is stored [D, page_size]
      } else {
        vp = v_win + ((size_t)(row0 + (s - S)) * Hkv + kvh) * D + d;
      }
      acc += pw * to_f32(*vp);
    }
  }
  s_red[tid] = acc;
  __syncthreads();
  if (tid < D) {
    float t = 0.f;
    for (int i = 0; i < nslice; ++i) t += s_red[i * D + tid];
    if (sizeof(T) == 2 && o_f16) ((bf16_t*)o)[((size_t)r * Hq + hq) * D + tid] = f32_to_f16_bits(t / denom);   // the consuming GEMM runs on half operands
    else o[((size_t)r * Hq + hq) * D + tid] = from_f32<T>(t / denom);
  }
}

template <int NW, bool SPLIT>
__global__ __launch_bounds__(NW * 64) void attn_flash_kernel(
    const bf16_t* __restrict__ q, int q_ld, int q_lo, const bf16_t* __restrict__ k_win, const bf16_t* __restrict__ vT_win,
    const bf16_t* __restrict__ k_pages, const bf16_t* __restrict__ v_pages, KvGeom g, Plan p, int Hq, int Z,
    int wpad, float scale_log2e, bf16_t* __restrict__ o, int o_ld, int o_lo, float* __restrict__ part_o,
    float* __restrict__ part_ml, int32_t* __restrict__ counters, int items, const uint4* __restrict__ pf, size_t pf_n16) {
  extern __shared__ float smem[];
  if ((int)blockIdx.z >= items) {
    // Workgroups behind the attention's own: they read the weights of the GEMMs that follow this launch, so that
    // those find them in the memory-side cache.  The attention is bound by dependent round trips, not by
    // bandwidth, and leaves most compute units and nearly all of the HBM time of its launch unused.
    const size_t nwg = (size_t)(gridDim.z - items) * gridDim.y * gridDim.x;
    const size_t wg = ((size_t)(blockIdx.z - items) * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    const size_t per = (pf_n16 + nwg - 1) / nwg, b0 = wg * per, b1 = min(pf_n16, b0 + per);
    for (size_t i = b0 + threadIdx.x; i < b1; i += (size_t)8 * NW * 64) {
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = pf[min(i + (size_t)u * NW * 64, b1 - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u) asm volatile("" ::"v"(v[u].x), "v"(v[u].y), "v"(v[u].z), "v"(v[u].w));
    }
    return;
  }
  attn_flash_body<NW, SPLIT, false>(q, q_ld, q_lo, k_win, vT_win, k_pages, v_pages, g, p, Hq, Z, wpad, scale_log2e, o, o_ld,
                                    o_lo, part_o, part_ml, counters, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.y, smem);
}


// Floats needed for `entries` split partials (one per (sequence, KV head, query tile, split)).
size_t attention_flash_partial_floats(size_t entries) { return entries * (32 * FA_D + 64); }

// q_tiles = ceil(3 B grp / 32); Z key splits of 8 wavefronts each.  `counters` holds one zeroed
// arrival counter per (sequence, KV head, query tile); the last split to arrive merges.
void launch_attention_flash(hipStream_t st, const void* q, int q_ld, int q_lo, const void* k_win, const void* vT_win,
                            const void* k_pages_layer, const void* v_pages_layer, const KvGeom& g, const Plan& p,
                            int N, int Hq, int q_tiles, int Z, int wpad, void* o, int o_ld, int o_lo, float* part,
                            int32_t* counters, const void* prefetch, size_t prefetch_bytes, int prefetch_wgs) {
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)g.head_dim);
  const int items = N * g.n_kv_heads;
  float* part_o = part;
  float* part_ml = part + (size_t)items * q_tiles * Z * 32 * FA_D;
  // extra slabs of Z * q_tiles workgroups that only read `prefetch` (see the kernel)
  const int slabs = prefetch && prefetch_bytes >= 16 ? std::min(65535 - items, (prefetch_wgs + Z * q_tiles - 1) / (Z * q_tiles)) : 0;
  const uint4* pf = (const uint4*)prefetch;
  const size_t pf_n16 = slabs > 0 ? prefetch_bytes / 16 : 0;
  if (q_lo)
    S2D2_LAUNCH((attn_flash_kernel<8, true>), dim3(Z, q_tiles, items + slabs), dim3(8 * 64), fa_lds(8), st,
                       (const bf16_t*)q, q_ld, q_lo, (const bf16_t*)k_win, (const bf16_t*)vT_win,
                       (const bf16_t*)k_pages_layer, (const bf16_t*)v_pages_layer, g, p, Hq, Z, wpad, scale_log2e,
                       (bf16_t*)o, o_ld, o_lo, part_o, part_ml, counters, items, pf, pf_n16);
  else
    S2D2_LAUNCH((attn_flash_kernel<8, false>), dim3(Z, q_tiles, items + slabs), dim3(8 * 64), fa_lds(8), st,
                       (const bf16_t*)q, q_ld, q_lo, (const bf16_t*)k_win, (const bf16_t*)vT_win,
                       (const bf16_t*)k_pages_layer, (const bf16_t*)v_pages_layer, g, p, Hq, Z, wpad, scale_log2e,
                       (bf16_t*)o, o_ld, o_lo, part_o, part_ml, counters, items, pf, pf_n16);
}

#ifdef S2D2_KERNEL_TIMING
__global__ void attn_ts_copy_kernel(unsigned long long* out) { if (threadIdx.x < 64) out[threadIdx.x] = g_attn_ts[threadIdx.x]; }
void launch_attn_ts_copy(hipStream_t st, void* out) { S2D2_LAUNCH(attn_ts_copy_kernel, dim3(1), dim3(64), 0, st, (unsigned long long*)out); }
#else
void launch_attn_ts_copy(hipStream_t, void*) {}
#endif

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
void launch_fill_i32(hipStream_t st, int32_t* p, int n, int32_t v) {
  S2D2_LAUNCH(fill_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n, v);
}

// Raises the dynamic-LDS limit of the kernels once (160 KB per workgroup on gfx950).
int attention_init() {
  hipError_t e = hipFuncSetAttribute((const void*)attn_generic_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_generic_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_flash_kernel<8, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fa_lds(8));
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)attn_flash_kernel<8, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fa_lds(8));
  return e == hipSuccess ? 0 : -1;
}

size_t attention_generic_lds_bytes(const KvGeom& g, int max_window_rows) {
  const size_t keys = (size_t)g.max_pages_per_seq * g.page_size + max_window_rows;
  return (g.head_dim + 264 + keys) * sizeof(float);
}

void launch_attention_generic(hipStream_t st, int dtype, const void* q, const void* k_win, const void* v_win,
                              const void* k_pages_layer, const void* v_pages_layer, const KvGeom& g,
                              const Plan& p, int rows_cap, int Hq, void* o, size_t lds_bytes, int o_f16) {
  const float scale = 1.0f / sqrtf((float)g.head_dim);
  dim3 grid(rows_cap, Hq), block(256);
  if (dtype == S2D2_BF16) {
    S2D2_LAUNCH(attn_generic_kernel<bf16_t>, grid, block, lds_bytes, st, (const bf16_t*)q,
                       (const bf16_t*)k_win, (const bf16_t*)v_win, (const bf16_t*)k_pages_layer,
                       (const bf16_t*)v_pages_layer, g, p, Hq, (bf16_t*)o, scale, o_f16);
  } else {
    S2D2_LAUNCH(attn_generic_kernel<float>, grid, block, lds_bytes, st, (const float*)q,
                       (const float*)k_win, (const float*)v_win, (const float*)k_pages_layer,
                       (const float*)v_pages_layer, g, p, Hq, (float*)o, scale, 0);
  }
}

}  // namespace s2d2
