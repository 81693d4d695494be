// Internal declarations shared by the HIP translation units of libs2d2.  Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

namespace s2d2 {

// Measurement aid: when the profiling scope has armed an event pair, the next kernel launch is made with
// hipExtLaunchKernelGGL, which stamps the two events with the dispatch's own start and end times (what a
// kernel trace reports); otherwise an ordinary launch.
extern thread_local hipEvent_t g_prof_start, g_prof_stop;
#define S2D2_LAUNCH(kernel, grid, block, lds, st, ...)                                                          \
  do {                                                                                                         \
    if (s2d2::g_prof_start) {                                                                                  \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, st, s2d2::g_prof_start, s2d2::g_prof_stop, 0, __VA_ARGS__); \
      s2d2::g_prof_start = nullptr;                                                                            \
    } else {                                                                                                   \
      hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);                                           \
    }                                                                                                          \
  } while (0)

typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
// Load of data that is read once per launch (the weight stream): the non-temporal hint keeps it from displacing
// what is re-read (activations, K/V of a short prefix, partial sums) from the caches.  On the 1.7B-shaped step it
// took 4.5 % off (3.14 -> 3.00 ms), most of it in the latency-bound kernels between the GEMMs.
template <typename T>
__device__ __forceinline__ T ld_stream(const T* p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// High- and low-order bf16 planes of a float: v ~= hi + lo with 16 significant bits.
__device__ __forceinline__ void split_bf16(float v, bf16_t& hi, bf16_t& lo) {
  hi = f32_to_bf16(v);
  lo = f32_to_bf16(v - bf16_to_f32(hi));
}
// ---- how an activation row that feeds a GEMM is stored -------------------------------------------------------
// Every such row comes with a "low-plane offset" next to its pointer:
//   0        one plane of bf16 values                                   (8 significant bits)
//   > 0      two planes, [hi | lo] that many elements apart: v ~= hi + lo (16 significant bits; every weight
//            operand is multiplied with both: twice the matrix instructions)
//   LO_F16   one plane of IEEE half values (11 significant bits); the GEMMs then run the f16 MFMA against weights
//            whose packed copy was converted from bf16 to half (exact for |w| >= 2^-17; below that the absolute
//            error is at most 2^-25), at the same matrix rate as bf16 and half the instructions of two planes.
constexpr int LO_F16 = -1;
enum OperandMode { OPM_BF16 = 0, OPM_BF16X2 = 1, OPM_F16 = 2 };
__host__ __device__ inline int operand_mode(int lo) { return lo == LO_F16 ? OPM_F16 : (lo > 0 ? OPM_BF16X2 : OPM_BF16); }
__device__ __forceinline__ bf16_t f32_to_f16_bits(float f) {   // round to nearest even, as 16 raw bits
  const _Float16 h = (_Float16)f;
  return __builtin_bit_cast(bf16_t, h);
}
// Stores one value / four consecutive values of such a row at p (the lo plane, if there is one, at p + lo).
__device__ __forceinline__ void act_store1(bf16_t* p, int lo, float v) {
  if (lo == LO_F16) { *p = f32_to_f16_bits(v); return; }
  bf16_t hi, l;
  split_bf16(v, hi, l);
  *p = hi;
  if (lo > 0) p[lo] = l;
}
__device__ __forceinline__ void act_pack4(int lo, float a, float b, float c, float d, uint2& first, uint2& second) {
  if (lo == LO_F16) {
    first = make_uint2((uint32_t)f32_to_f16_bits(a) | ((uint32_t)f32_to_f16_bits(b) << 16),
                       (uint32_t)f32_to_f16_bits(c) | ((uint32_t)f32_to_f16_bits(d) << 16));
    second = first;
    return;
  }
  bf16_t hi[4], l[4];
  split_bf16(a, hi[0], l[0]);
  split_bf16(b, hi[1], l[1]);
  split_bf16(c, hi[2], l[2]);
  split_bf16(d, hi[3], l[3]);
  first = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
  second = make_uint2((uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16));
}
__device__ __forceinline__ void act_store4(bf16_t* p, int lo, float a, float b, float c, float d) {
  uint2 f, s2;
  act_pack4(lo, a, b, c, d, f, s2);
  *(uint2*)p = f;
  if (lo > 0) *(uint2*)(p + lo) = s2;
}
// One MFMA 16x16x32 on 16-byte operand fragments in either operand type.
template <int OPM>
__device__ __forceinline__ f32x4_t mfma_16x16x32(const u32x4_t& a, const u32x4_t& b, const f32x4_t& c) {
  if (OPM == OPM_F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// Device-coherent accesses (agent scope, relaxed: write-through stores, loads that bypass the non-coherent
// caches) for data that workgroups of one launch hand to each other.  The producer waits for its stores
// (s_waitcnt) before it signals; no cache-wide fence is involved.
__device__ __forceinline__ uint4 ld16_coh(const void* p) {
  const uint64_t* q = (const uint64_t*)p;
  const uint64_t a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const uint64_t b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_uint4((uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32));
}
__device__ __forceinline__ void st8_coh(void* p, uint2 v) {
  __hip_atomic_store((uint64_t*)p, (uint64_t)v.x | ((uint64_t)v.y << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st2_coh(bf16_t* p, bf16_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st4f_coh(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld4f_coh(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st16f_coh(float* p, float a, float b, float c, float d) {
  uint64_t* q = (uint64_t*)p;
  __hip_atomic_store(q, (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(q + 1, (uint64_t)__float_as_uint(c) | ((uint64_t)__float_as_uint(d) << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return f32_to_bf16(x); }

// ---- device-resident description of one forward's window rows (built by the plan kernel) ----
// Rows of all sequences are packed back to back; the rows of sequence n are
// [seq_row0[n], seq_row0[n] + seq_rows[n]).  Row r attends to every cached position of its
// sequence, to the window rows [row_lo[r], row_hi[r]) and to itself.
struct Plan {
  int32_t* counts;      // [0] = number of window rows, [1] = number of logit rows
  int32_t* row_token;   // [rows_cap]
  int32_t* row_pos;     // [rows_cap] absolute position (RoPE phase)
  int32_t* row_seq;     // [rows_cap]
  int32_t* row_lo;      // [rows_cap]
  int32_t* row_hi;      // [rows_cap]
  int32_t* logit_src;   // [logit_cap] window row whose hidden state feeds logit row k
  int32_t* logit_seq;   // [logit_cap]
  int32_t* logit_idx;   // [logit_cap] block index scored by logit row k
  int32_t* seq_row0;    // [max_batch]
  int32_t* seq_rows;    // [max_batch]
  int32_t* seq_lead;    // [max_batch] leading causal rows before C_t (carry + pending)
  int32_t* seq_j;       // [max_batch] first masked block index (B if none)
  int32_t* seq_L;       // [max_batch] |C_t|
  int32_t vocab;        // token ids outside [0, vocab) in the caller's state are read as [MASK]
};

struct KvGeom {
  const int32_t* page_table;
  const int32_t* seq_len;
  int32_t n_pages, page_size, max_pages_per_seq;
  int32_t n_kv_heads, head_dim;
};

enum GemmEpilogue {
  EPI_STORE_F32 = 0,   // out_f32[m, n] = acc                       (ldo floats per row)
  EPI_ADD_F32 = 1,     // out_f32[m, n] += acc                      (residual stream)
  EPI_SWIGLU = 2,      // out_act[m, n] = silu(acc_gate) * acc_up   (W holds [2, N, K])
};

// plan.hip
void launch_plan(hipStream_t st, int verify /* 0 draft, 1 verifier, 2 block completion, 3 causal block completion of blocks the carry cannot take */, int shifted /* right-shifted model */,
                 int N, int B, int mask_id, int ar_mask,
                 const int32_t* seq_len, const int32_t* pos0, const int32_t* block,
                 const int32_t* carry, const int32_t* xhat, const Plan& p, int32_t* logit_row_of,
                 int32_t* span_start, int32_t* span_len, int32_t* stage_row0, int32_t* stage_lead,
                 const int32_t* active, int32_t* status,
                 float* clear_a = nullptr, float* clear_b = nullptr /* verifier: [N, B] outputs zeroed for every position */);
void launch_kv_append(hipStream_t st, int dtype, int n_layers, int N, int rows_cap, const KvGeom& g,
                      void* k_pages, void* v_pages, const void* k_stage, const void* v_stage,
                      const int32_t* stage_row0, const int32_t* stage_lead, const int32_t* span_len,
                      const int32_t* n_accept, int32_t* seq_len, int32_t* status, int B,
                      int hold_back /* 1: the last drafted token has no staged row */);
void launch_block_advance(hipStream_t st, int N, int B, int mask_id, const int32_t* seq_len,
                          int32_t* pos0, int32_t* block, int32_t* carry, uint32_t* step_dev, int32_t* status);
void launch_commit_threshold(hipStream_t st, int N, int B, int32_t* block, const int32_t* xhat,
                             const uint64_t* unmask);

// elementwise.hip
void launch_embed(hipStream_t st, int dtype, const void* embed, int d, const Plan& p, int rows_cap, float* h);
// out[r] = rmsnorm(h[src(r)]) * gain as `dtype`; src = gather[r] if gather else r; rows from *count.
void launch_rmsnorm(hipStream_t st, int dtype, const float* h, const float* gain, int d, float eps,
                    const int32_t* count, const int32_t* gather, int rows_cap, void* out);
void launch_rope_split(hipStream_t st, int dtype, const float* qkv, const Plan& p, int rows_cap, int Hq,
                       int Hkv, int D, float theta, void* q_out, void* k_out, void* v_out, void* vT_out, int wpad);

// gemm.hip : Y[m, n] = sum_k X[m, k] * W[n, k], X and W in `dtype`, fp32 accumulation.
void launch_gemm(hipStream_t st, int dtype, GemmEpilogue epi, const void* X, int ldx, const void* W, int K,
                 int N, const int32_t* m_count, int m_cap, void* out, int ldo);

// gemm_stream.hip : packed-weight streaming GEMM with fused prologue / epilogue (bf16)
enum StreamEpilogue { SEPI_STORE_F32 = 0, SEPI_ADD_F32 = 1, SEPI_SWIGLU = 2, SEPI_QKV_ROPE = 3 };
enum StreamPrologue { SPRO_BF16 = 0, SPRO_BF16S = 1 };  // S: scale the result by 1/rms from partial sums
enum GemmGrouping { GROUP_NONE = 0, GROUP_GATHER = 1, GROUP_SCATTER = 2 };  // expert-grouped rows (tile kernel only)
struct GemmStreamArgs {
  const uint4* Wp;          // packed weights [NT][KT][64] x 16 bytes
  const uint4* Wp2;         // second matrix (up projection) for SEPI_SWIGLU
  int32_t NT, KT, N, K;
  const int32_t* m_count;   // device: number of valid rows
  int32_t m_hint;           // host: rows the caller expects (0 = unknown); only steers the choice of launch shape
  const bf16_t* X;          // activations [*, ldx] (for SPRO_BF16S: h * gain, not yet divided by the rms)
  int32_t ldx;
  int32_t x_lo;             // low-plane offset of X's rows (0: one bf16 plane, > 0: two planes, LO_F16: half values)
  const int32_t* gather;    // optional row indices into X / ss_part
  const float* ss_part;     // SPRO_BF16S: [*, ss_stride] partial sums of squares of the residual rows
  int32_t ss_stride, ss_count;
  float eps;
  void* out;
  int32_t ldo;
  int32_t out_lo;           // SEPI_SWIGLU: low-plane offset of the output rows (as x_lo)
  // SEPI_ADD_F32 extras (all optional): operand of the next norm and its partial sums of squares
  bf16_t* xg_out;           // [*, xg_ld]
  int32_t xg_ld, xg_lo;     // row stride and low-plane offset (as x_lo) of xg_out
  const float* gain_next;   // [N]
  float* ss_out;            // [*, ss_stride], entry nt of a row = this tile's share
  // SEPI_QKV_ROPE
  const float2* rope_cs;    // [rows, D/2] (cos, sin)
  int32_t Hq, Hkv, D, wpad;
  int32_t q_ld, q_lo;       // row stride of q_out and offset of its low-order plane (0: single plane)
  bf16_t* q_out;
  bf16_t* k_out;
  bf16_t* v_out;
  bf16_t* vT_out;
  bf16_t* k16_out;          // optional second copy of the window's keys as IEEE half, same layout as k_out (read by the
                            // attention kernel for wide windows in the half mode instead of the bf16 rows)
  int32_t win_f16;          // vT_out holds IEEE half instead of bf16 (same reader)
  const int32_t* row_seq;
  const int32_t* seq_row0;
  // expert-grouped rows (tile kernel): row tile t covers sorted slots [tile_row0[t], +tile_rows[t]) of expert
  // tile_expert[t]; sorted[s] = token * top_k + slot.  GROUP_GATHER reads X row sorted[s] / top_k and writes
  // row s; GROUP_SCATTER reads X row s and writes row sorted[s], scaled by route_w[sorted[s]].
  int32_t grouped, top_k;
  const int32_t* n_tiles;
  const int32_t* tile_expert;
  const int32_t* tile_row0;
  const int32_t* tile_rows;
  const int32_t* sorted;
  const float* route_w;
  size_t expert_stride;     // uint4 elements between the packed matrices of consecutive experts
  // split K of the tile kernel: fp32 partials (64 KB per workgroup) and one arrival counter per tile
  float* tile_partials;
  int32_t* tile_counters;
  int32_t tile_partial_cap, tile_counter_cap;
  int32_t merge_spins;      // set by the tile kernel's launcher: polls a K split waits for the other splits of its tile before it gives its share up
  int32_t stream_k;         // set by the tile kernel's launcher: 0, or the row tiles of a launch that runs 3/2 tiles per workgroup
  int32_t xcd_order;        // set by the tile kernel's launcher: tiles are re-dealt so that the row tiles of a column share an XCD
  int32_t split_xcd;        // set by the tile kernel's launcher: K split z runs on the XCDs x with x % splits == z
  int32_t coop_wgs;         // compute units: a launch of at most that many workgroups of the tile kernel is resident at once (0: unknown)
  // streaming kernel, paired K split of the residual-add GEMM: pair_cap x 256 (value, tag) words, zero between
  // launches; *pair_status is set when a bounded wait ran out
  unsigned long long* pair_buf;
  int32_t* pair_status;
  int32_t pair_cap;
};
size_t packed_weight_bytes(int N, int K);
void launch_pack_weight(hipStream_t st, const void* W, int N, int K, int rope_pairs, int D, void* out, int to_f16 /* convert bf16 -> half */);
void launch_rope_table(hipStream_t st, const Plan& p, int rows_cap, int D, float theta, void* cs);
void launch_embed_norm(hipStream_t st, const void* embed, int d, const Plan& p, int rows_cap, const float* gain,
                       float* h, void* xg, int xg_ld, int xg_lo, float* ss, int ss_stride,
                       void* rope_cs /* [rows, D/2] (cos, sin), may be NULL */, int D, float theta);
void launch_gemm_stream(hipStream_t st, int kind, const GemmStreamArgs& a, int m_cap);
// gemm_tile.hip : 128 x 256 LDS-tiled kernel on the same packed weights and argument block
void launch_gemm_tile(hipStream_t st, int kind, int pro, const GemmStreamArgs& a, int row_tiles);

// moe.hip
void launch_moe_route(hipStream_t st, const float* logits, int E, int top_k, const int32_t* m_count, int rows_cap,
                      int32_t* choice, float* route_w);
void launch_moe_group(hipStream_t st, int E, int top_k, const int32_t* m_count, const int32_t* choice,
                      int32_t* sorted, int32_t* tile_expert, int32_t* tile_row0, int32_t* tile_rows, int32_t* n_tiles,
                      int tile_cap);
void launch_moe_combine(hipStream_t st, const float* y, int d, int top_k, const int32_t* m_count, int rows_cap,
                        float* h, void* xg, int xg_ld, int xg_lo, const float* gain_next, float* ss, int ss_stride);
void launch_moe_copy_choices(hipStream_t st, const int32_t* src, int32_t* dst, int layers, int per_layer_src,
                             int per_layer_dst);

// attention.hip
void launch_attention_generic(hipStream_t st, int dtype, const void* q, const void* k_win, const void* v_win,
                              const void* k_pages_layer, const void* v_pages_layer, const KvGeom& g,
                              const Plan& p, int rows_cap, int Hq, void* o, size_t lds_bytes, int o_f16 /* bf16 models: write o as half values */);
int attention_init();
size_t attention_flash_partial_floats(size_t entries);
void launch_attention_flash(hipStream_t st, const void* q, int q_ld, int q_lo, const void* k_win, const void* vT_win,
                            const void* k_pages_layer, const void* v_pages_layer, const KvGeom& g, const Plan& p,
                            int N, int Hq, int q_tiles, int Z, int wpad, void* o, int o_ld, int o_lo, float* part,
                            int32_t* counters, const void* prefetch, size_t prefetch_bytes, int prefetch_wgs);
// Several query tiles per (sequence, KV head): one workgroup shares each K / V tile among them.
int attention_wide_init();
int attention_wide_nw(int q_tiles);
int attention_wide_pt_cap(const KvGeom& g, int Z);
size_t attention_wide_lds_bytes(int pt_cap);
void launch_attention_wide(hipStream_t st, const void* q, int q_ld, int q_lo, const void* k_win, const void* vT_win,
                           const void* k_pages_layer, const void* v_pages_layer, const KvGeom& g, const Plan& p, int N,
                           int Hq, int q_tiles, int Z, int wpad, void* o, int o_ld, int o_lo, float* part,
                           size_t part_entries, int32_t* counters);
void launch_fill_i32(hipStream_t st, int32_t* p, int n, int32_t v);
void launch_attn_ts_copy(hipStream_t st, void* out);   // timing build only
void launch_wide_ts_copy(hipStream_t st, void* out);   // timing build only
void launch_tile_ts_copy(hipStream_t st, void* out);   // timing build only
void launch_stream_ts_copy(hipStream_t st, void* out); // timing build only
size_t attention_generic_lds_bytes(const KvGeom& g, int max_window_rows);

// vocab.hip
struct VocabWs {
  float* part;       // [rows_cap_logits, chunks, 8] partial statistics
  int32_t chunks;
};
int vocab_chunks(int V);
struct VocabSample {   // sampling mode of SampleFromLogits: proposals drawn from softmax(logits / temperature)
  bool sample;
  float temperature;
  uint64_t seed;
  uint32_t step;
  const uint32_t* step_dev;
};
void launch_vocab_draft(hipStream_t st, const float* logits, int V, const int32_t* count, int rows_cap,
                        const VocabWs& ws, const int32_t* logit_seq, const int32_t* logit_idx, int B,
                        int32_t* xhat, float* p, float* lse, float* margin, float* entropy_n, const VocabSample& sm);
void launch_vocab_score(hipStream_t st, const float* logits, int V, const int32_t* count, int rows_cap,
                        const VocabWs& ws, const int32_t* logit_seq, const int32_t* logit_idx, int B,
                        const int32_t* token, float* q, float* lse, float inv_t);
void launch_draft_finish(hipStream_t st, int N, int B, int mask_id, float tau, const int32_t* block,
                         int32_t* xhat, float* p, float* lse, float* margin, float* entropy_n,
                         uint64_t* unmask, int32_t* n_hi);
void launch_accept(hipStream_t st, int N, int B, int V, uint64_t seed, uint32_t step, const uint32_t* step_dev,
                   float gamma, int resample, float inv_t, const int32_t* span_start, const int32_t* span_len,
                   const float* logits_d, const int32_t* row_of_d, const float* logits_v,
                   const int32_t* row_of_v, const int32_t* xhat, const float* p, const float* lse_d,
                   const float* q, const float* lse_v, int32_t* block, int32_t* n_accept, int32_t* n_commit,
                   int32_t* resampled, float* u_used, const int32_t* active, float* tile_scratch /* accept_tile_floats, may be NULL */,
                   int32_t* arrivals /* [max_batch], zero between launches, may be NULL */);
size_t accept_tile_floats(int max_batch, int V);
// Limits of the accept step that takes its scratch from a device array of the library, and the per-device address
// of that array's two parts (looked up on the first call on a device; the device must be current).  0 on success.
constexpr int ACCEPT_STATIC_MAX_BATCH = 128, ACCEPT_STATIC_MAX_VOCAB = 1 << 18;
int accept_static_scratch(float** tiles, int32_t** arrivals);

}  // namespace s2d2
