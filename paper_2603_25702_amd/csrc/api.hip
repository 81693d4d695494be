// C ABI of libs2d2: argument validation, workspace carving, and the launch sequence of the
// draft / verifier forward.  See include/s2d2.h for the contract of every entry point.
#include "../../include/s2d2.h"
#include "../../include/s2d2_aux.h"
#include "s2d2_internal.h"

#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <stdarg.h>
#include <vector>
#include <algorithm>

using namespace s2d2;

static thread_local char g_err[512] = "";
namespace s2d2 { thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr; }
namespace s2d2 {   // defined in plan.hip (takes a type of the public header)
void launch_route(hipStream_t st, int N, int B, const s2d2_route_params& rp, const int32_t* span_start,
                  const int32_t* span_len, const float* margin, const float* entropy_n, const int32_t* n_hi,
                  const uint64_t* unmask, int32_t* hysteresis, int32_t* do_verify, float* khat, float* score,
                  uint64_t* unmask_fallback);
}

static int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

struct s2d2_ctx {
  s2d2_model_desc desc;
  s2d2_weights w;
  s2d2_layer_weights* layers;
  int32_t max_batch, max_block, rows_cap, logit_cap;
  hipStream_t stream;
  uint8_t* ws;
  size_t ws_bytes;
  // carved workspace
  Plan plan;
  int32_t* tmp_count;
  float* h;
  void* a;
  float* qkv;
  void* qbuf;
  void* obuf;
  void* ffn;
  void* af;
  void* kwin;
  void* vwin;
  void* vT_win;      // [max_batch, Hkv, D, wpad] key-minor V of the window (MFMA attention)
  void* kwin16;      // [rows_cap, Hkv, D] the window's keys as half values (wide attention kernel in the half mode)
  float* attn_part;  // split-key partial outputs
  size_t attn_part_entries;
  int32_t* attn_counters;  // arrival counters of the split-key merge, zero between launches
  int32_t attn_groups;
  int32_t wpad, attn_zmax;
  VocabWs vws;
  float2* rope_cs;   // [rows_cap, D/2] cos / sin of the window rows
  int32_t* zeros_i32;  // [max_batch] zeros (never written)
  float* ss;         // [rows_cap, d/16] partial sums of squares of the residual rows (split RMSNorm)
  // packed bf16 weights (streaming GEMM); null when the caller gave no packed buffer
  struct PackedLayer { const uint4 *wqkv, *wo, *wg, *wu, *wdown, *router, *eg, *eu, *ed; };
  // MoE scratch
  float* router_logits;   // [rows_cap, E]
  int32_t* moe_choice;    // [n_layers, rows_cap * top_k] experts chosen in the last forward
  float* moe_w;           // [rows_cap * top_k] renormalised routing weights
  int32_t* moe_sorted;    // [rows_cap * top_k]
  int32_t *moe_tile_expert, *moe_tile_row0, *moe_tile_rows, *moe_n_tiles;
  int32_t moe_tile_cap;
  void* moe_act;          // [rows_cap * top_k, d_expert]
  float* moe_y;           // [rows_cap * top_k, d_model]
  PackedLayer* pk;
  const uint4* pk_unembed;
  int32_t* dev_status;       // sticky device-side failure words ([1]: a bounded wait of the paired K split ran out)
  uint64_t* ts_scratch;      // clock stamps of the timing build
  int n_cus;                 // compute units of the device
  float* tile_partials;      // split-K partials of the tiled GEMM, TILE_PARTIAL_CAP x 64 KB
  int32_t* tile_counters;    // TILE_COUNTER_CAP arrival counters, zero between launches
  float* accept_tiles;       // [max_batch, vocabulary tiles] residual tile sums shared by the workgroups of a sequence
  int32_t* accept_arrive;    // [max_batch] their arrival counters, zero between launches
  unsigned long long* pair_buf;   // PAIR_CAP x 256 (value, tag) words of the streaming GEMM's paired K split, zero between launches
  int32_t prefetch_wgs;     // workgroups of the narrow attention launch that read the next two GEMMs' weights ahead
  int wide_wgs;             // workgroups the split choice of the wide attention kernel aims for
  // profiling (measurement aid)
  bool prof_on;
  int32_t prof_cap;
  struct ProfRec { int cls, sub; double bytes, flops; hipEvent_t a, b; };
  std::vector<ProfRec>* prof;
  std::vector<hipEvent_t>* prof_pool;
};

namespace {

constexpr int TILE_PARTIAL_CAP = 4096, TILE_COUNTER_CAP = 4096, PAIR_CAP = 512;

struct Carver {
  uint8_t* base;
  size_t off = 0;
  template <typename T> T* take(size_t n) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? (T*)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

int elt_size(int dtype) { return dtype == S2D2_BF16 ? 2 : 4; }
// planes the workspace reserves per GEMM input row (bf16 models: room for two, whatever the operand mode)
int act_planes(const s2d2_model_desc& d) { return d.dtype == S2D2_BF16 ? 2 : 1; }
// how the packed-weight GEMMs of a bf16 model take their inputs (s2d2_model_desc.act_planes)
int operand_mode_of(const s2d2_model_desc& d) {
  if (d.act_planes == 1) return OPM_BF16;
  if (d.act_planes == 2) return OPM_BF16X2;
  return OPM_F16;   // 0 (default) and 3
}

int32_t check_desc(const s2d2_model_desc* d) {
  if (!d) return fail(S2D2_EINVAL, "model description is NULL");
  if (d->dtype != S2D2_F32 && d->dtype != S2D2_BF16) return fail(S2D2_EINVAL, "dtype must be S2D2_F32 or S2D2_BF16");
  if (d->n_layers < 1 || d->n_layers > 4096 || d->d_model < 32 || d->d_model > 65536 || d->vocab < 2) return fail(S2D2_EINVAL, "n_layers (1-4096), d_model (32-65536) or vocab out of range");
  if (d->n_q_heads < 1 || d->n_q_heads > 1024 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads) return fail(S2D2_EINVAL, "n_q_heads must be a positive multiple of n_kv_heads, at most 1024");
  if (d->d_ffn > (1 << 20) || d->d_expert > (1 << 20)) return fail(S2D2_EINVAL, "d_ffn and d_expert must not exceed 1048576");
  if (d->head_dim != 32 && d->head_dim != 64 && d->head_dim != 128 && d->head_dim != 256) return fail(S2D2_EINVAL, "head_dim must be 32, 64, 128 or 256");
  const int kq = d->dtype == S2D2_BF16 ? 32 : 16;  // one MFMA fragment must not straddle the end of K
  if (d->d_model % kq || (d->n_q_heads * d->head_dim) % kq) return fail(S2D2_EINVAL, "d_model and Hq*D must be multiples of %d", kq);
  if (d->n_experts == 0) {
    if (d->d_ffn < kq || d->d_ffn % kq) return fail(S2D2_EINVAL, "d_ffn must be a positive multiple of %d", kq);
    if (d->top_k || d->d_expert) return fail(S2D2_EINVAL, "top_k and d_expert must be 0 for a dense model");
  } else {
    if (d->n_experts < 0 || d->n_experts > 256 || d->top_k < 1 || d->top_k > d->n_experts || d->top_k > 64 ||
        d->d_expert < kq || d->d_expert % kq)
      return fail(S2D2_EINVAL, "MoE shape out of range (n_experts <= 256, top_k <= min(64, n_experts), d_expert a multiple of %d)", kq);
    if (d->dtype != S2D2_BF16) return fail(S2D2_EINVAL, "MoE models must be bf16");
    if (d->d_ffn) return fail(S2D2_EINVAL, "d_ffn must be 0 for a MoE model");
  }
  if (d->mask_id < 0 || d->mask_id >= d->vocab) return fail(S2D2_EINVAL, "mask_id outside the vocabulary");
  if (d->act_planes < 0 || d->act_planes > 3) return fail(S2D2_EINVAL, "act_planes must be 0, 1, 2 or 3");
  if (d->right_shifted != 0 && d->right_shifted != 1) return fail(S2D2_EINVAL, "right_shifted must be 0 or 1");
  if (d->vocab > 8192 * 256) return fail(S2D2_EINVAL, "vocab above 2097152 is not supported");
  if (!(d->rope_theta > 1.0f) || !(d->rms_eps >= 0.0f)) return fail(S2D2_EINVAL, "rope_theta must exceed 1 and rms_eps be non-negative");
  return S2D2_OK;
}

int32_t check_limits(int32_t max_batch, int32_t max_block) {
  if (max_batch < 1 || max_batch > 1024) return fail(S2D2_EINVAL, "max_batch must be in [1, 1024]");
  if (max_block < 1 || max_block > S2D2_MAX_BLOCK) return fail(S2D2_EINVAL, "max_block must be in [1, %d]", S2D2_MAX_BLOCK);
  return S2D2_OK;
}

// Lays the workspace out; with base == NULL only measures.
size_t carve(s2d2_ctx* c, uint8_t* base) {
  const s2d2_model_desc& d = c->desc;
  Carver cv{base};
  const size_t R = c->rows_cap, LR = c->logit_cap, NB = c->max_batch;
  const size_t es = elt_size(d.dtype);
  c->plan.counts = cv.take<int32_t>(8);
  c->plan.vocab = d.vocab;
  c->tmp_count = cv.take<int32_t>(8);
  c->plan.row_token = cv.take<int32_t>(R);
  c->plan.row_pos = cv.take<int32_t>(R);
  c->plan.row_seq = cv.take<int32_t>(R);
  c->plan.row_lo = cv.take<int32_t>(R);
  c->plan.row_hi = cv.take<int32_t>(R);
  c->plan.logit_src = cv.take<int32_t>(LR);
  c->plan.logit_seq = cv.take<int32_t>(LR);
  c->plan.logit_idx = cv.take<int32_t>(LR);
  c->plan.seq_row0 = cv.take<int32_t>(NB);
  c->plan.seq_rows = cv.take<int32_t>(NB);
  c->plan.seq_lead = cv.take<int32_t>(NB);
  c->plan.seq_j = cv.take<int32_t>(NB);
  c->plan.seq_L = cv.take<int32_t>(NB);
  c->h = cv.take<float>(R * d.d_model);
  const size_t P = act_planes(d);
  c->a = cv.take<uint8_t>(R * d.d_model * es * P);
  c->qkv = cv.take<float>(R * (size_t)(d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim);
  c->qbuf = cv.take<uint8_t>(R * (size_t)d.n_q_heads * d.head_dim * es * act_planes(d));
  c->obuf = cv.take<uint8_t>(R * (size_t)d.n_q_heads * d.head_dim * es * P);
  c->ffn = cv.take<uint8_t>(R * (size_t)d.d_ffn * es * P);
  c->af = cv.take<uint8_t>(LR * (size_t)d.d_model * es);
  c->kwin = cv.take<uint8_t>(R * (size_t)d.n_kv_heads * d.head_dim * es);
  c->vwin = cv.take<uint8_t>(R * (size_t)d.n_kv_heads * d.head_dim * es);
  c->wpad = (3 * c->max_block + 31) / 32 * 32;
  c->attn_zmax = 64;
  c->vT_win = cv.take<uint8_t>(NB * (size_t)d.n_kv_heads * d.head_dim * c->wpad * es);
  c->kwin16 = cv.take<uint8_t>(d.dtype == S2D2_BF16 ? R * (size_t)d.n_kv_heads * d.head_dim * 2 : 0);
  {
    const int q_tiles = (3 * c->max_block * (d.n_q_heads / d.n_kv_heads) + 31) / 32;
    // Z * items * q_tiles < 512 * 8 + items * q_tiles by the choice of Z in forward()
    c->attn_part_entries = 4096 + NB * d.n_kv_heads * q_tiles;
    c->attn_part = cv.take<float>(attention_flash_partial_floats(c->attn_part_entries));
    c->attn_groups = (int32_t)(NB * d.n_kv_heads * q_tiles);
    c->attn_counters = cv.take<int32_t>(c->attn_groups);
  }
  c->rope_cs = cv.take<float2>(R * (size_t)(d.head_dim / 2));
  c->ss = cv.take<float>(R * (size_t)((d.d_model + 15) / 16));
  c->zeros_i32 = cv.take<int32_t>(NB);
  if (d.n_experts > 0) {
    const size_t RK = R * (size_t)d.top_k;
    c->router_logits = cv.take<float>(R * (size_t)d.n_experts);
    c->moe_choice = cv.take<int32_t>((size_t)d.n_layers * RK);
    c->moe_w = cv.take<float>(RK);
    c->moe_sorted = cv.take<int32_t>(RK);
    c->moe_tile_cap = (int32_t)(RK / 128 + d.n_experts + 1);
    c->moe_tile_expert = cv.take<int32_t>(c->moe_tile_cap);
    c->moe_tile_row0 = cv.take<int32_t>(c->moe_tile_cap);
    c->moe_tile_rows = cv.take<int32_t>(c->moe_tile_cap);
    c->moe_n_tiles = cv.take<int32_t>(8);
    c->moe_act = cv.take<uint8_t>(RK * (size_t)d.d_expert * es * P);
    c->moe_y = cv.take<float>(RK * (size_t)d.d_model);
  }
  if (d.dtype == S2D2_BF16) {
    c->tile_partials = cv.take<float>((size_t)TILE_PARTIAL_CAP * 16384);
    c->tile_counters = cv.take<int32_t>(TILE_COUNTER_CAP);
    c->pair_buf = cv.take<unsigned long long>((size_t)PAIR_CAP * 256);
  }
  c->dev_status = cv.take<int32_t>(64);
  c->ts_scratch = cv.take<uint64_t>(1024);
  c->vws.chunks = vocab_chunks(d.vocab);
  c->vws.part = cv.take<float>(LR * (size_t)c->vws.chunks * 8);
  c->accept_tiles = cv.take<float>(accept_tile_floats(c->max_batch, d.vocab));
  c->accept_arrive = cv.take<int32_t>(c->max_batch);
  return (cv.off + 255) & ~(size_t)255;
}

// Arms the event pair of the next kernel launch (S2D2_LAUNCH) and books it under a class.  A scope that holds
// several launches times the first one.
struct ProfScope {
  ProfScope(s2d2_ctx* c, int cls, double bytes, double flops = 0.0, int sub = -1) {
    if (!c->prof_on || (int32_t)c->prof->size() >= c->prof_cap) return;
    hipEvent_t a = (*c->prof_pool)[2 * c->prof->size()], b = (*c->prof_pool)[2 * c->prof->size() + 1];
    c->prof->push_back({cls, sub, bytes, flops, a, b});
    g_prof_start = a;
    g_prof_stop = b;
  }
  ~ProfScope() { g_prof_start = nullptr; }
};

size_t packed_total_bytes(const s2d2_model_desc& d) {
  if (d.dtype != S2D2_BF16) return 0;
  const int HqD = d.n_q_heads * d.head_dim, qkv_n = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
  size_t per = packed_weight_bytes(qkv_n, d.d_model) + packed_weight_bytes(d.d_model, HqD);
  if (d.n_experts > 0)
    per += packed_weight_bytes(d.n_experts, d.d_model) +
           (size_t)d.n_experts * (2 * packed_weight_bytes(d.d_expert, d.d_model) + packed_weight_bytes(d.d_model, d.d_expert));
  else
    per += 2 * packed_weight_bytes(d.d_ffn, d.d_model) + packed_weight_bytes(d.d_model, d.d_ffn);
  return per * d.n_layers + packed_weight_bytes(d.vocab, d.d_model);
}

int32_t check_launch(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(S2D2_ELAUNCH, "%s: %s", what, hipGetErrorString(e));
  return S2D2_OK;
}

int32_t check_kv(const s2d2_ctx* c, const s2d2_kv_view* kv) {
  if (!kv || !kv->k_pages || !kv->v_pages || !kv->page_table || !kv->seq_len) return fail(S2D2_EINVAL, "kv view or one of its pointers is NULL");
  if (kv->n_pages < 1 || kv->page_size < 1 || kv->max_pages_per_seq < 1) return fail(S2D2_EINVAL, "kv view: n_pages, page_size and max_pages_per_seq must be positive");
  if (((uintptr_t)kv->k_pages | (uintptr_t)kv->v_pages) & 15) return fail(S2D2_EINVAL, "kv pages must be 16-byte aligned");
  return S2D2_OK;
}

int32_t check_state(const s2d2_ctx* c, const s2d2_block_state* st, int32_t N, int32_t B) {
  if (!c) return fail(S2D2_EINVAL, "ctx is NULL");
  if (N < 1 || N > c->max_batch) return fail(S2D2_EINVAL, "N=%d outside [1, max_batch=%d]", N, c->max_batch);
  if (B < 1 || B > c->max_block) return fail(S2D2_EINVAL, "B=%d outside [1, max_block=%d]", B, c->max_block);
  if (!st || !st->block_tokens || !st->block_pos0 || !st->carry_tokens) return fail(S2D2_EINVAL, "block state or one of its pointers is NULL");
  return S2D2_OK;
}

KvGeom geom(const s2d2_ctx* c, const s2d2_kv_view* kv) {
  return KvGeom{kv->page_table, kv->seq_len, kv->n_pages, kv->page_size, kv->max_pages_per_seq,
                c->desc.n_kv_heads, c->desc.head_dim};
}

// One forward over the planned window rows; K/V of every window row go to k_stage/v_stage
// ([n_layers, rows_cap, Hkv, D]) if given, else to a one-layer scratch.
int32_t forward(s2d2_ctx* c, const s2d2_kv_view* kv, int32_t N, int32_t B, void* k_stage, void* v_stage, float* logits) {
  const s2d2_model_desc& d = c->desc;
  const int dt = d.dtype, R = (k_stage ? 3 : 2) * N * B, LR = N * B, es = elt_size(dt);  // row bounds of this call (draft: carry + block)
  const int HqD = d.n_q_heads * d.head_dim, qkv_n = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
  hipStream_t st = c->stream;
  const KvGeom g = geom(c, kv);
  // MFMA flash attention for bf16 / head_dim 128 / pages that hold whole 8-key groups; else the generic kernel
  const bool flash = dt == S2D2_BF16 && d.head_dim == 128 && kv->page_size % 8 == 0;
  const int q_tiles = ((k_stage ? 3 : 2) * B * (d.n_q_heads / d.n_kv_heads) + 31) / 32;   // 32-row query tiles of this call's windows
  int Z = 1;
  // several query tiles per (sequence, KV head): the kernel that shares K / V tiles among them
  bool wide = flash && q_tiles >= 2 && (kv->page_size & (kv->page_size - 1)) == 0;
  if (flash) {
    // Splits until there are ~512 workgroups or a wavefront is down to one 32-key tile; the last
    // split to finish merges, so extra splits cost one atomic, not a launch.
    const int cap_tiles = (kv->max_pages_per_seq * kv->page_size + 31) / 32;
    const int groups = N * d.n_kv_heads * q_tiles;
    const int want = (512 + groups - 1) / groups;
    Z = std::max(1, std::min(std::min(want, (cap_tiles + 7) / 8), c->attn_zmax));
    if (wide) {
      // one workgroup per (sequence, KV head, group of query tiles, split); a split keeps at least 4 key tiles
      const int wg = N * d.n_kv_heads * ((q_tiles + 7) / 8);
      Z = std::max(1, std::min((c->wide_wgs + wg - 1) / wg, std::min((cap_tiles + 3) / 4, c->attn_zmax)));
      while (Z > 1 && ((size_t)Z * N * d.n_kv_heads * q_tiles > c->attn_part_entries ||
                       attention_wide_lds_bytes(attention_wide_pt_cap(g, Z)) > 160 * 1024)) --Z;
      if (attention_wide_lds_bytes(attention_wide_pt_cap(g, Z)) > 160 * 1024) wide = false, Z = 1;
    }
  }
  const size_t lds = flash ? 0 : attention_generic_lds_bytes(g, 3 * B);
  if (lds > 160 * 1024) return fail(S2D2_ENOSPC, "attention needs %zu bytes of LDS for max_pages_per_seq*page_size=%d keys (limit 163840)", lds, kv->max_pages_per_seq * kv->page_size);
  const size_t stage_layer = (size_t)c->rows_cap * d.n_kv_heads * d.head_dim * es;
  const size_t page_layer = (size_t)kv->n_pages * d.n_kv_heads * kv->page_size * d.head_dim * es;
  const int32_t* n_rows = c->plan.counts;
  const bool fused = c->pk != nullptr;
  const int ss_stride = (d.d_model + 15) / 16;
  // rows a fresh block gives: N*B draft rows, 2*N*B verifier rows (more only with carried or pending committed tokens)
  const int m_hint = (k_stage ? 2 : 1) * N * B;
  const double fr = 2.0 * m_hint, fl = 2.0 * N * B;   // flops per weight element: layer GEMMs, unembedding (method's flops, one plane)
  auto sk = [&](GemmStreamArgs& x) {   // split-K buffers of the tiled GEMM, expected rows
    x.m_hint = x.m_count == c->plan.counts + 1 ? N * B : m_hint;   // (logit rows: one per masked position)
    x.tile_partials = c->tile_partials; x.tile_counters = c->tile_counters;
    x.tile_partial_cap = TILE_PARTIAL_CAP; x.tile_counter_cap = TILE_COUNTER_CAP; x.coop_wgs = c->n_cus;
    x.pair_buf = c->pair_buf; x.pair_status = c->dev_status + 1; x.pair_cap = PAIR_CAP;
  };
  // GEMM inputs: one plane of half values, or P bf16 planes per row ([hi | lo]); the low-plane offsets say which
  // (0: one bf16 plane; LO_F16: half).  The plain kernels (no packed copy, or the generic attention) use one bf16 plane.
  // (the generic attention kernel reads and writes single planes: two-plane models then run on their high plane)
  const int mode = operand_mode_of(d);
  const int opm = !fused ? OPM_BF16 : (flash || mode == OPM_F16 ? mode : OPM_BF16);
  const int P = opm == OPM_BF16X2 ? 2 : 1;
  auto lo_of = [&](int width) { return opm == OPM_F16 ? LO_F16 : (P == 2 ? width : 0); };
  const int ld_a = P * d.d_model, lo_a = lo_of(d.d_model);
  const int ld_o = P * HqD, lo_o = lo_of(HqD);
  const int ld_f = P * d.d_ffn, lo_f = lo_of(d.d_ffn);
  const int ld_e = P * d.d_expert, lo_e = lo_of(d.d_expert);
  // queries stay bf16 (the attention kernels multiply them with the cache's bf16 keys): hi + lo planes unless the
  // model asked for single bf16 planes
  // model asked for single bf16 planes; the kernel for wide windows takes them as half values in the half mode
  // (it converts the keys and values on their way into LDS)
  const bool q_f16 = fused && wide && opm == OPM_F16;
  const int PQ = fused && flash && opm != OPM_BF16 && !q_f16 ? 2 : 1;
  const int ld_q = PQ * HqD, lo_q = q_f16 ? LO_F16 : (PQ == 2 ? HqD : 0);
  if (fused) { ProfScope ps(c, 3, 0.0); launch_embed_norm(st, c->w.embed, d.d_model, c->plan, R, c->layers[0].norm1, c->h, c->a, ld_a, lo_a, c->ss, ss_stride, c->rope_cs, d.head_dim, d.rope_theta); }
  else { ProfScope ps(c, 3, 0.0); launch_embed(st, dt, c->w.embed, d.d_model, c->plan, R, c->h); }
  for (int l = 0; l < d.n_layers; ++l) {
    const s2d2_layer_weights& L = c->layers[l];
    void* kw = k_stage ? (uint8_t*)k_stage + l * stage_layer : c->kwin;
    void* vw = v_stage ? (uint8_t*)v_stage + l * stage_layer : c->vwin;
    if (fused) {
      GemmStreamArgs a{};
      a.Wp = c->pk[l].wqkv; a.NT = qkv_n / 16; a.KT = d.d_model / 32; a.N = qkv_n; a.K = d.d_model;
      a.m_count = n_rows; a.X = (const bf16_t*)c->a; a.ldx = ld_a; a.x_lo = lo_a; a.ss_part = c->ss; a.ss_stride = ss_stride;
      a.ss_count = l == 0 ? 1 : ss_stride; a.eps = d.rms_eps;
      a.rope_cs = c->rope_cs; a.Hq = d.n_q_heads; a.Hkv = d.n_kv_heads; a.D = d.head_dim; a.wpad = c->wpad;
      a.q_out = (bf16_t*)c->qbuf; a.q_ld = ld_q; a.q_lo = lo_q; a.k_out = (bf16_t*)kw; a.v_out = (bf16_t*)vw; a.vT_out = flash ? (bf16_t*)c->vT_win : nullptr;
      a.row_seq = c->plan.row_seq; a.seq_row0 = c->plan.seq_row0;
      if (q_f16) { a.k16_out = (bf16_t*)c->kwin16; a.win_f16 = 1; }
      ProfScope ps(c, 0, (double)qkv_n * d.d_model * es, fr * qkv_n * d.d_model, 4);
      sk(a); launch_gemm_stream(st, SEPI_QKV_ROPE, a, R);
    } else {
      { ProfScope ps(c, 3, 0.0); launch_rmsnorm(st, dt, c->h, L.norm1, d.d_model, d.rms_eps, n_rows, nullptr, R, c->a); }
      { ProfScope ps(c, 0, (double)qkv_n * d.d_model * es, fr * qkv_n * d.d_model, 4); launch_gemm(st, dt, EPI_STORE_F32, c->a, d.d_model, L.wqkv, d.d_model, qkv_n, n_rows, R, c->qkv, qkv_n); }
      { ProfScope ps(c, 3, 0.0); launch_rope_split(st, dt, c->qkv, c->plan, R, d.n_q_heads, d.n_kv_heads, d.head_dim, d.rope_theta, c->qbuf, kw, vw, flash ? c->vT_win : nullptr, c->wpad); }
    }
    const void* kp = (const uint8_t*)kv->k_pages + l * page_layer;
    const void* vp = (const uint8_t*)kv->v_pages + l * page_layer;
    if (flash) {
      ProfScope ps(c, 1, 0.0);
      if (wide)
        launch_attention_wide(st, c->qbuf, fused ? ld_q : HqD, fused ? lo_q : 0, q_f16 ? c->kwin16 : kw, c->vT_win, kp, vp, g, c->plan, N, d.n_q_heads, q_tiles, Z, c->wpad, c->obuf, ld_o, lo_o, c->attn_part, c->attn_part_entries, c->attn_counters);
      else
      {
        // Narrow windows of a few sequences: the launch is a chain of dependent round trips on a fraction of the
        // compute units.  Workgroups behind the attention's own read the weights of the next two GEMMs (the packed
        // matrices of a layer lie one behind the other: wo, gate, up, down) into the memory-side cache meanwhile.
        size_t ahead = 0;
        if (fused && d.n_experts == 0 && R <= 32 && Z * q_tiles * N * d.n_kv_heads <= 128)
          ahead = packed_weight_bytes(d.d_model, HqD) + 2 * packed_weight_bytes(d.d_ffn, d.d_model);
        launch_attention_flash(st, c->qbuf, fused ? ld_q : HqD, fused ? lo_q : 0, kw, c->vT_win, kp, vp, g, c->plan, N, d.n_q_heads, q_tiles, Z, c->wpad, c->obuf, ld_o, lo_o, c->attn_part, c->attn_counters,
                               ahead ? c->pk[l].wo : nullptr, ahead, c->prefetch_wgs);
      }
    } else {
      ProfScope ps(c, 1, 0.0);
      launch_attention_generic(st, dt, c->qbuf, kw, vw, kp, vp, g, c->plan, R, d.n_q_heads, c->obuf, lds, opm == OPM_F16);
    }
    if (fused) {
      GemmStreamArgs a{};
      a.m_count = n_rows;
      a.Wp = c->pk[l].wo; a.NT = d.d_model / 16; a.KT = HqD / 32; a.N = d.d_model; a.K = HqD;
      a.X = (const bf16_t*)c->obuf; a.ldx = ld_o; a.x_lo = lo_o; a.out = c->h; a.ldo = d.d_model;
      a.xg_out = (bf16_t*)c->a; a.xg_ld = ld_a; a.xg_lo = lo_a; a.gain_next = L.norm2; a.ss_out = c->ss; a.ss_stride = ss_stride;
      { ProfScope ps(c, 0, (double)d.d_model * HqD * es, fr * d.d_model * HqD, 5); sk(a); launch_gemm_stream(st, SEPI_ADD_F32, a, R); }
      const float* gain_after = l + 1 < d.n_layers ? c->layers[l + 1].norm1 : c->w.norm_f;
      if (d.n_experts == 0) {
        GemmStreamArgs b{};
        b.m_count = n_rows;
        b.Wp = c->pk[l].wg; b.Wp2 = c->pk[l].wu; b.NT = d.d_ffn / 16; b.KT = d.d_model / 32; b.N = d.d_ffn; b.K = d.d_model;
        b.X = (const bf16_t*)c->a; b.ldx = ld_a; b.x_lo = lo_a; b.ss_part = c->ss; b.ss_stride = ss_stride; b.ss_count = ss_stride;
        b.eps = d.rms_eps; b.out = c->ffn; b.ldo = ld_f; b.out_lo = lo_f;
        { ProfScope ps(c, 0, 2.0 * d.d_ffn * d.d_model * es, fr * 2.0 * d.d_ffn * d.d_model, 6); sk(b); launch_gemm_stream(st, SEPI_SWIGLU, b, R); }
        GemmStreamArgs e{};
        e.m_count = n_rows;
        e.Wp = c->pk[l].wdown; e.NT = d.d_model / 16; e.KT = d.d_ffn / 32; e.N = d.d_model; e.K = d.d_ffn;
        e.X = (const bf16_t*)c->ffn; e.ldx = ld_f; e.x_lo = lo_f; e.out = c->h; e.ldo = d.d_model;
        e.xg_out = (bf16_t*)c->a; e.xg_ld = ld_a; e.xg_lo = lo_a; e.gain_next = gain_after; e.ss_out = c->ss; e.ss_stride = ss_stride;
        { ProfScope ps(c, 0, (double)d.d_model * d.d_ffn * es, fr * d.d_model * d.d_ffn, 7); sk(e); launch_gemm_stream(st, SEPI_ADD_F32, e, R); }
      } else {
        // MoE FFN: router -> top-k -> group by expert -> grouped gate/up + SwiGLU -> grouped down -> combine
        const int E = d.n_experts, Fe = d.d_expert, tk = d.top_k;
        int32_t* choice = c->moe_choice + (size_t)l * c->rows_cap * tk;
        GemmStreamArgs r{};
        r.m_count = n_rows;
        r.Wp = c->pk[l].router; r.NT = (E + 15) / 16; r.KT = d.d_model / 32; r.N = E; r.K = d.d_model;
        r.X = (const bf16_t*)c->a; r.ldx = ld_a; r.x_lo = lo_a; r.ss_part = c->ss; r.ss_stride = ss_stride; r.ss_count = ss_stride;
        r.eps = d.rms_eps; r.out = c->router_logits; r.ldo = E;
        { ProfScope ps(c, 0, (double)E * d.d_model * es, fr * E * d.d_model); sk(r); launch_gemm_stream(st, SEPI_STORE_F32, r, R); }
        { ProfScope ps(c, 3, 0.0); launch_moe_route(st, c->router_logits, E, tk, n_rows, R, choice, c->moe_w); }
        { ProfScope ps(c, 3, 0.0); launch_moe_group(st, E, tk, n_rows, choice, c->moe_sorted, c->moe_tile_expert,
                                                     c->moe_tile_row0, c->moe_tile_rows, c->moe_n_tiles, c->moe_tile_cap); }
        const int tile_cap = std::min(c->moe_tile_cap, R * tk / 128 + E + 1);
        GemmStreamArgs b{};
        b.grouped = GROUP_GATHER; b.top_k = tk; b.n_tiles = c->moe_n_tiles; b.tile_expert = c->moe_tile_expert;
        b.tile_row0 = c->moe_tile_row0; b.tile_rows = c->moe_tile_rows; b.sorted = c->moe_sorted; b.route_w = c->moe_w;
        b.expert_stride = packed_weight_bytes(Fe, d.d_model) / 16;
        b.Wp = c->pk[l].eg; b.Wp2 = c->pk[l].eu; b.NT = Fe / 16; b.KT = d.d_model / 32; b.N = Fe; b.K = d.d_model;
        b.X = (const bf16_t*)c->a; b.ldx = ld_a; b.x_lo = lo_a; b.ss_part = c->ss; b.ss_stride = ss_stride; b.ss_count = ss_stride;
        b.eps = d.rms_eps; b.out = c->moe_act; b.ldo = ld_e; b.out_lo = lo_e;
        { ProfScope ps(c, 0, 2.0 * E * (double)Fe * d.d_model * es, fr * tk * 2.0 * Fe * d.d_model, 6); launch_gemm_tile(st, SEPI_SWIGLU, SPRO_BF16S, b, tile_cap); }
        GemmStreamArgs e{};
        e.grouped = GROUP_SCATTER; e.top_k = tk; e.n_tiles = c->moe_n_tiles; e.tile_expert = c->moe_tile_expert;
        e.tile_row0 = c->moe_tile_row0; e.tile_rows = c->moe_tile_rows; e.sorted = c->moe_sorted; e.route_w = c->moe_w;
        e.expert_stride = packed_weight_bytes(d.d_model, Fe) / 16;
        e.Wp = c->pk[l].ed; e.NT = d.d_model / 16; e.KT = Fe / 32; e.N = d.d_model; e.K = Fe;
        e.X = (const bf16_t*)c->moe_act; e.ldx = ld_e; e.x_lo = lo_e; e.out = c->moe_y; e.ldo = d.d_model;
        { ProfScope ps(c, 0, (double)E * d.d_model * Fe * es, fr * tk * (double)d.d_model * Fe, 7); launch_gemm_tile(st, SEPI_STORE_F32, SPRO_BF16, e, tile_cap); }
        { ProfScope ps(c, 3, 0.0); launch_moe_combine(st, c->moe_y, d.d_model, tk, n_rows, R, c->h, c->a, ld_a, lo_a, gain_after, c->ss, ss_stride); }
      }
    } else {
      { ProfScope ps(c, 0, (double)d.d_model * HqD * es, fr * d.d_model * HqD, 5); launch_gemm(st, dt, EPI_ADD_F32, c->obuf, HqD, L.wo, HqD, d.d_model, n_rows, R, c->h, d.d_model); }
      { ProfScope ps(c, 3, 0.0); launch_rmsnorm(st, dt, c->h, L.norm2, d.d_model, d.rms_eps, n_rows, nullptr, R, c->a); }
      { ProfScope ps(c, 0, 2.0 * d.d_ffn * d.d_model * es, fr * 2.0 * d.d_ffn * d.d_model, 6); launch_gemm(st, dt, EPI_SWIGLU, c->a, d.d_model, L.wgu, d.d_model, d.d_ffn, n_rows, R, c->ffn, d.d_ffn); }
      { ProfScope ps(c, 0, (double)d.d_model * d.d_ffn * es, fr * d.d_model * d.d_ffn, 7); launch_gemm(st, dt, EPI_ADD_F32, c->ffn, d.d_ffn, L.wdown, d.d_ffn, d.d_model, n_rows, R, c->h, d.d_model); }
    }
  }
  const int32_t* n_logit = c->plan.counts + 1;
  if (fused) {
    GemmStreamArgs a{};
    a.Wp = c->pk_unembed; a.NT = (d.vocab + 15) / 16; a.KT = d.d_model / 32; a.N = d.vocab; a.K = d.d_model;
    a.m_count = n_logit; a.X = (const bf16_t*)c->a; a.ldx = ld_a; a.x_lo = lo_a; a.gather = c->plan.logit_src;
    a.ss_part = c->ss; a.ss_stride = ss_stride; a.ss_count = ss_stride; a.eps = d.rms_eps;
    a.out = logits; a.ldo = d.vocab;
    ProfScope ps(c, 0, (double)d.vocab * d.d_model * es, fl * d.vocab * d.d_model, 8);
    sk(a); launch_gemm_stream(st, SEPI_STORE_F32, a, LR);
  } else {
    { ProfScope ps(c, 3, 0.0); launch_rmsnorm(st, dt, c->h, c->w.norm_f, d.d_model, d.rms_eps, n_logit, c->plan.logit_src, LR, c->af); }
    { ProfScope ps(c, 0, (double)d.vocab * d.d_model * es, fl * d.vocab * d.d_model, 8); launch_gemm(st, dt, EPI_STORE_F32, c->af, d.d_model, c->w.unembed, d.d_model, d.vocab, n_logit, LR, logits, d.vocab); }
  }
  return check_launch("forward");
}

__global__ void set_i32_kernel(int32_t* p, int32_t v) { *p = v; }

}  // namespace

extern "C" {

const char* s2d2_last_error(void) { return g_err; }
const char* s2d2_version(void) { return "s2d2-gfx950 0.1"; }

int64_t s2d2_stage_rows(int32_t max_batch, int32_t max_block) {
  if (check_limits(max_batch, max_block)) return S2D2_EINVAL;
  return (int64_t)3 * max_batch * max_block;
}

int64_t s2d2_workspace_bytes(const s2d2_model_desc* desc, int32_t max_batch, int32_t max_block) {
  int32_t rc = check_desc(desc);
  if (rc) return rc;
  rc = check_limits(max_batch, max_block);
  if (rc) return rc;
  s2d2_ctx tmp;
  memset(&tmp, 0, sizeof(tmp));
  tmp.desc = *desc;
  tmp.max_batch = max_batch;
  tmp.max_block = max_block;
  tmp.rows_cap = 3 * max_batch * max_block;
  tmp.logit_cap = max_batch * max_block;
  return (int64_t)carve(&tmp, nullptr);
}

int64_t s2d2_packed_bytes(const s2d2_model_desc* desc) {
  const int32_t rc = check_desc(desc);
  if (rc) return rc;
  return (int64_t)packed_total_bytes(*desc);
}

int32_t s2d2_create(const s2d2_model_desc* desc, const s2d2_weights* weights, int32_t max_batch,
                    int32_t max_block, void* stream, void* workspace, size_t workspace_bytes, void* packed,
                    size_t packed_bytes, s2d2_ctx** out) {
  if (!out) return fail(S2D2_EINVAL, "out is NULL");
  *out = nullptr;
  int32_t rc = check_desc(desc);
  if (rc) return rc;
  rc = check_limits(max_batch, max_block);
  if (rc) return rc;
  if (!weights || !weights->embed || !weights->unembed || !weights->norm_f || !weights->layers) return fail(S2D2_EINVAL, "weights or one of its pointers is NULL");
  for (int l = 0; l < desc->n_layers; ++l) {
    const s2d2_layer_weights& L = weights->layers[l];
    if (!L.norm1 || !L.wqkv || !L.wo || !L.norm2) return fail(S2D2_EINVAL, "layer %d: attention weights missing", l);
    if (desc->n_experts == 0 && (!L.wgu || !L.wdown)) return fail(S2D2_EINVAL, "layer %d: FFN weights missing", l);
    if (desc->n_experts > 0 && (!L.router || !L.e_wgu || !L.e_wdown)) return fail(S2D2_EINVAL, "layer %d: MoE weights missing", l);
    if (((uintptr_t)L.wqkv | (uintptr_t)L.wo | (uintptr_t)L.wgu | (uintptr_t)L.wdown | (uintptr_t)L.router |
         (uintptr_t)L.e_wgu | (uintptr_t)L.e_wdown) & 15) return fail(S2D2_EINVAL, "layer %d: weights must be 16-byte aligned", l);
  }
  if (((uintptr_t)weights->embed | (uintptr_t)weights->unembed) & 15) return fail(S2D2_EINVAL, "embed/unembed must be 16-byte aligned");
  if (!workspace || ((uintptr_t)workspace & 255)) return fail(S2D2_EINVAL, "workspace is NULL or not 256-byte aligned");
  const int64_t need = s2d2_workspace_bytes(desc, max_batch, max_block);
  if (need < 0) return (int32_t)need;
  if (workspace_bytes < (size_t)need) return fail(S2D2_ENOSPC, "workspace has %zu bytes, %lld needed", workspace_bytes, (long long)need);
  const bool use_packed = packed != nullptr && packed_total_bytes(*desc) > 0;
  if (desc->n_experts > 0 && !use_packed) return fail(S2D2_EINVAL, "MoE models need the packed weight buffer (s2d2_packed_bytes)");
  if (packed && ((uintptr_t)packed & 255)) return fail(S2D2_EINVAL, "packed buffer is not 256-byte aligned");
  if (use_packed && packed_bytes < packed_total_bytes(*desc)) return fail(S2D2_ENOSPC, "packed buffer has %zu bytes, %zu needed", packed_bytes, packed_total_bytes(*desc));

  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return fail(S2D2_EARCH, "no usable HIP device");
  }
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return fail(S2D2_EARCH, "device is %s, this library is built for gfx950", prop.gcnArchName);

  s2d2_ctx* c = (s2d2_ctx*)calloc(1, sizeof(s2d2_ctx));
  if (!c) return fail(S2D2_ENOSPC, "out of host memory");
  c->desc = *desc;
  c->w = *weights;
  c->layers = (s2d2_layer_weights*)malloc(sizeof(s2d2_layer_weights) * desc->n_layers);
  if (!c->layers) { free(c); return fail(S2D2_ENOSPC, "out of host memory"); }
  memcpy(c->layers, weights->layers, sizeof(s2d2_layer_weights) * desc->n_layers);
  c->w.layers = c->layers;
  c->max_batch = max_batch;
  c->n_cus = prop.multiProcessorCount;
  c->max_block = max_block;
  c->rows_cap = 3 * max_batch * max_block;
  c->logit_cap = max_batch * max_block;
  c->stream = (hipStream_t)stream;
  c->ws = (uint8_t*)workspace;
  c->ws_bytes = workspace_bytes;
  carve(c, c->ws);
  c->wide_wgs = 512;
  if (use_packed) {  // re-lay the projection weights out for the streaming GEMM (enqueued on the stream)
    const s2d2_model_desc& d = c->desc;
    const int HqD = d.n_q_heads * d.head_dim, qkv_n = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    c->pk = (s2d2_ctx::PackedLayer*)malloc(sizeof(s2d2_ctx::PackedLayer) * d.n_layers);
    uint8_t* p = (uint8_t*)packed;
    const int to_f16 = operand_mode_of(d) == OPM_F16;
    auto put = [&](const void* W, int N, int K, int rope) {
      const uint4* at = (const uint4*)p;
      launch_pack_weight(c->stream, W, N, K, rope, d.head_dim, p, to_f16);
      p += packed_weight_bytes(N, K);
      return at;
    };
    for (int l = 0; l < d.n_layers; ++l) {
      const s2d2_layer_weights& L = c->layers[l];
      c->pk[l].wqkv = put(L.wqkv, qkv_n, d.d_model, 1);
      c->pk[l].wo = put(L.wo, d.d_model, HqD, 0);
      if (d.n_experts == 0) {
        c->pk[l].wg = put(L.wgu, d.d_ffn, d.d_model, 0);
        c->pk[l].wu = put((const uint8_t*)L.wgu + (size_t)d.d_ffn * d.d_model * 2, d.d_ffn, d.d_model, 0);
        c->pk[l].wdown = put(L.wdown, d.d_model, d.d_ffn, 0);
      } else {  // experts: all gate matrices, then all up matrices, then all down matrices, each [E] packed copies
        const size_t mat = (size_t)d.d_expert * d.d_model * 2;
        c->pk[l].router = put(L.router, d.n_experts, d.d_model, 0);
        for (int e = 0; e < d.n_experts; ++e) {
          const uint4* at = put((const uint8_t*)L.e_wgu + (size_t)(2 * e) * mat, d.d_expert, d.d_model, 0);
          if (e == 0) c->pk[l].eg = at;
        }
        for (int e = 0; e < d.n_experts; ++e) {
          const uint4* at = put((const uint8_t*)L.e_wgu + (size_t)(2 * e + 1) * mat, d.d_expert, d.d_model, 0);
          if (e == 0) c->pk[l].eu = at;
        }
        for (int e = 0; e < d.n_experts; ++e) {
          const uint4* at = put((const uint8_t*)L.e_wdown + (size_t)e * mat, d.d_model, d.d_expert, 0);
          if (e == 0) c->pk[l].ed = at;
        }
      }
    }
    c->pk_unembed = put(c->w.unembed, d.vocab, d.d_model, 0);
    if (hipGetLastError() != hipSuccess) { free(c->pk); free(c->layers); free(c); return fail(S2D2_ELAUNCH, "weight packing failed to launch"); }
  }
  c->prefetch_wgs = 128;
  launch_fill_i32(c->stream, c->dev_status, 64, 0);
  launch_fill_i32(c->stream, c->attn_counters, c->attn_groups, 0);
  launch_fill_i32(c->stream, c->zeros_i32, c->max_batch, 0);
  launch_fill_i32(c->stream, c->accept_arrive, c->max_batch, 0);
  if (c->tile_counters) launch_fill_i32(c->stream, c->tile_counters, TILE_COUNTER_CAP, 0);
  if (c->pair_buf) launch_fill_i32(c->stream, (int32_t*)c->pair_buf, PAIR_CAP * 256 * 2, 0);
  if (accept_static_scratch(nullptr, nullptr)) { (void)hipGetLastError(); free(c->pk); free(c->layers); free(c); return fail(S2D2_ELAUNCH, "could not look up the device address of the library's scratch array"); }
  if (attention_init() || attention_wide_init()) { (void)hipGetLastError(); free(c->pk); free(c->layers); free(c); return fail(S2D2_ELAUNCH, "could not raise the LDS limit of the attention kernel"); }
  *out = c;
  return S2D2_OK;
}

int32_t s2d2_destroy(s2d2_ctx* ctx) {
  if (!ctx) return fail(S2D2_EINVAL, "ctx is NULL");
  if (ctx->prof_pool) {
    for (hipEvent_t e : *ctx->prof_pool) (void)hipEventDestroy(e);
    delete ctx->prof_pool;
    delete ctx->prof;
  }
  free(ctx->pk);
  free(ctx->layers);
  free(ctx);
  return S2D2_OK;
}

int32_t s2d2_set_stream(s2d2_ctx* ctx, void* stream) {
  if (!ctx) return fail(S2D2_EINVAL, "ctx is NULL");
  ctx->stream = (hipStream_t)stream;
  return S2D2_OK;
}

static int32_t check_params(const s2d2_params* p) {
  if (!p) return fail(S2D2_EINVAL, "params is NULL");
  if (p->mode != S2D2_GREEDY && p->mode != S2D2_SAMPLE) return fail(S2D2_EINVAL, "unknown drafting mode %d", p->mode);
  if (p->mode == S2D2_SAMPLE && !(p->temperature > 0.f)) return fail(S2D2_EINVAL, "sampling mode needs a positive temperature");
  if (!(p->gamma > 0.f)) return fail(S2D2_EINVAL, "gamma must be positive");
  if (!(p->tau >= 0.f)) return fail(S2D2_EINVAL, "tau must be non-negative");
  return S2D2_OK;
}

// 1 / T of the sampling mode; exactly 1 in greedy mode, where all probabilities are taken at temperature 1
static float inv_temperature(const s2d2_params* p) { return p->mode == S2D2_SAMPLE ? 1.0f / p->temperature : 1.0f; }

static int32_t check_draft_out(const s2d2_draft_out* o) {
  if (!o || !o->logits || !o->logit_row_of || !o->xhat || !o->p || !o->lse || !o->margin || !o->entropy_n ||
      !o->unmask || !o->n_hi || !o->span_start || !o->span_len)
    return fail(S2D2_EINVAL, "draft output or one of its pointers is NULL");
  if ((uintptr_t)o->logits & 15) return fail(S2D2_EINVAL, "draft logits must be 16-byte aligned");
  return S2D2_OK;
}

static int32_t check_verify_out(const s2d2_verify_out* o) {
  if (!o || !o->logits_ver || !o->logit_row_of || !o->q || !o->lse_ver || !o->k_stage || !o->v_stage ||
      !o->stage_row0 || !o->stage_lead)
    return fail(S2D2_EINVAL, "verify output or one of its pointers is NULL");
  if (((uintptr_t)o->logits_ver | (uintptr_t)o->k_stage | (uintptr_t)o->v_stage) & 15) return fail(S2D2_EINVAL, "verify logits and K/V stage must be 16-byte aligned");
  return S2D2_OK;
}

int32_t s2d2_draft(s2d2_ctx* c, const s2d2_kv_view* kv, const s2d2_block_state* st, int32_t N, int32_t B,
                   const s2d2_params* prm, const s2d2_draft_out* out) {
  int32_t rc;
  if ((rc = check_state(c, st, N, B)) || (rc = check_kv(c, kv)) || (rc = check_params(prm)) || (rc = check_draft_out(out))) return rc;
  const s2d2_model_desc& d = c->desc;
  { ProfScope ps(c, 3, 0.0); launch_plan(c->stream, 0, d.right_shifted, N, B, d.mask_id, prm->ar_mask, kv->seq_len, st->block_pos0, st->block_tokens,
              st->carry_tokens, nullptr, c->plan, out->logit_row_of, out->span_start, out->span_len, nullptr, nullptr, nullptr, kv->status); }
  if ((rc = forward(c, kv, N, B, nullptr, nullptr, out->logits))) return rc;
  { ProfScope ps(c, 2, 0.0); launch_vocab_draft(c->stream, out->logits, d.vocab, c->plan.counts + 1, N * B, c->vws, c->plan.logit_seq,
                     c->plan.logit_idx, B, out->xhat, out->p, out->lse, out->margin, out->entropy_n,
                     VocabSample{prm->mode == S2D2_SAMPLE, prm->temperature, prm->seed, prm->step, prm->step_dev}); }
  { ProfScope ps(c, 2, 0.0); launch_draft_finish(c->stream, N, B, d.mask_id, prm->tau, st->block_tokens, out->xhat, out->p, out->lse,
                      out->margin, out->entropy_n, out->unmask, out->n_hi); }
  return check_launch("s2d2_draft");
}

int32_t s2d2_verify(s2d2_ctx* c, const s2d2_kv_view* kv, const s2d2_block_state* st, int32_t N, int32_t B,
                    const s2d2_params* prm, const s2d2_draft_out* draft, const s2d2_verify_out* out) {
  int32_t rc;
  if ((rc = check_state(c, st, N, B)) || (rc = check_kv(c, kv)) || (rc = check_params(prm)) ||
      (rc = check_draft_out(draft)) || (rc = check_verify_out(out)))
    return rc;
  const s2d2_model_desc& d = c->desc;
  { ProfScope ps(c, 3, 0.0); launch_plan(c->stream, 1, d.right_shifted, N, B, d.mask_id, 1, kv->seq_len, st->block_pos0, st->block_tokens, st->carry_tokens,
              draft->xhat, c->plan, out->logit_row_of, nullptr, nullptr, out->stage_row0, out->stage_lead, prm->active, kv->status,
              out->q, out->lse_ver); }
  if ((rc = forward(c, kv, N, B, out->k_stage, out->v_stage, out->logits_ver))) return rc;
  { ProfScope ps(c, 2, 0.0); launch_vocab_score(c->stream, out->logits_ver, d.vocab, c->plan.counts + 1, N * B, c->vws, c->plan.logit_seq,
                     c->plan.logit_idx, B, draft->xhat, out->q, out->lse_ver, inv_temperature(prm)); }
  return check_launch("s2d2_verify");
}

int32_t s2d2_accept(s2d2_ctx* c, const s2d2_block_state* st, int32_t N, int32_t B, const s2d2_params* prm,
                    const s2d2_draft_out* draft, const s2d2_verify_out* ver, const s2d2_accept_out* out) {
  int32_t rc;
  if ((rc = check_state(c, st, N, B)) || (rc = check_params(prm)) || (rc = check_draft_out(draft)) ||
      (rc = check_verify_out(ver)))
    return rc;
  if (!out || !out->n_accept || !out->n_commit || !out->resampled || !out->u_used) return fail(S2D2_EINVAL, "accept output or one of its pointers is NULL");
  { ProfScope ps(c, 2, 0.0); launch_accept(c->stream, N, B, c->desc.vocab, prm->seed, prm->step, prm->step_dev, prm->gamma, prm->resample,
                inv_temperature(prm), draft->span_start, draft->span_len, draft->logits, draft->logit_row_of, ver->logits_ver,
                ver->logit_row_of, draft->xhat, draft->p, draft->lse, ver->q, ver->lse_ver, st->block_tokens,
                out->n_accept, out->n_commit, out->resampled, out->u_used, prm->active, c->accept_tiles, c->accept_arrive); }
  return check_launch("s2d2_accept");
}

int32_t s2d2_accept_static(void* stream, int32_t vocab, const s2d2_block_state* st, int32_t N, int32_t B,
                           const s2d2_params* prm, const s2d2_draft_out* draft, const s2d2_verify_out* ver,
                           const s2d2_accept_out* out) {
  int32_t rc;
  if (N < 1 || N > ACCEPT_STATIC_MAX_BATCH) return fail(S2D2_ENOSPC, "s2d2_accept_static: N=%d outside [1, %d] (the library's own scratch holds %d sequences; use s2d2_accept with a workspace)", N, ACCEPT_STATIC_MAX_BATCH, ACCEPT_STATIC_MAX_BATCH);
  if (vocab < 2 || vocab > ACCEPT_STATIC_MAX_VOCAB) return fail(S2D2_ENOSPC, "s2d2_accept_static: vocab=%d outside [2, %d] (size of the library's own scratch; use s2d2_accept with a workspace)", vocab, ACCEPT_STATIC_MAX_VOCAB);
  if (B < 1 || B > S2D2_MAX_BLOCK) return fail(S2D2_EINVAL, "B=%d outside [1, %d]", B, S2D2_MAX_BLOCK);
  if (!st || !st->block_tokens) return fail(S2D2_EINVAL, "block state or its block_tokens is NULL");
  if ((rc = check_params(prm)) || (rc = check_draft_out(draft)) || (rc = check_verify_out(ver))) return rc;
  if (!out || !out->n_accept || !out->n_commit || !out->resampled || !out->u_used) return fail(S2D2_EINVAL, "accept output or one of its pointers is NULL");
  float* tiles = nullptr;
  int32_t* arrivals = nullptr;
  if (accept_static_scratch(&tiles, &arrivals)) return fail(S2D2_ELAUNCH, "s2d2_accept_static: could not look up the device address of the library's scratch array");
  hipStream_t s = (hipStream_t)stream;
  // the array keeps what the last call left: the arrival counters must start at zero (a fill kernel, no memset node)
  launch_fill_i32(s, arrivals, N, 0);
  launch_accept(s, N, B, vocab, prm->seed, prm->step, prm->step_dev, prm->gamma, prm->resample, inv_temperature(prm),
                draft->span_start, draft->span_len, draft->logits, draft->logit_row_of, ver->logits_ver, ver->logit_row_of,
                draft->xhat, draft->p, draft->lse, ver->q, ver->lse_ver, st->block_tokens, out->n_accept, out->n_commit,
                out->resampled, out->u_used, prm->active, tiles, arrivals);
  return check_launch("s2d2_accept_static");
}

int32_t s2d2_kv_append(s2d2_ctx* c, const s2d2_kv_view* kv, int32_t N, int32_t B, const s2d2_draft_out* draft,
                       const s2d2_verify_out* ver, const int32_t* n_accept) {
  int32_t rc;
  if (!c) return fail(S2D2_EINVAL, "ctx is NULL");
  if (N < 1 || N > c->max_batch || B < 1 || B > c->max_block) return fail(S2D2_EINVAL, "N or B outside the limits given at create");
  if ((rc = check_kv(c, kv)) || (rc = check_draft_out(draft)) || (rc = check_verify_out(ver))) return rc;
  if (!n_accept) return fail(S2D2_EINVAL, "n_accept is NULL");
  const KvGeom g = geom(c, kv);
  { ProfScope ps(c, 3, 0.0); launch_kv_append(c->stream, c->desc.dtype, c->desc.n_layers, N, c->rows_cap, g, kv->k_pages, kv->v_pages,
                   ver->k_stage, ver->v_stage, ver->stage_row0, ver->stage_lead, draft->span_len, n_accept,
                   kv->seq_len, kv->status, B, c->desc.right_shifted); }
  return check_launch("s2d2_kv_append");
}

int32_t s2d2_block_complete(s2d2_ctx* c, const s2d2_kv_view* kv, const s2d2_block_state* st, int32_t N, int32_t B,
                            const s2d2_verify_out* scratch, int32_t causal) {
  int32_t rc;
  if ((rc = check_state(c, st, N, B)) || (rc = check_kv(c, kv)) || (rc = check_verify_out(scratch))) return rc;
  const s2d2_model_desc& d = c->desc;
  if (d.right_shifted) return fail(S2D2_EINVAL, "s2d2_block_complete is not defined for right-shifted models (their cache lags one token)");
  if (causal != 0 && causal != 1) return fail(S2D2_EINVAL, "causal must be 0 or 1");
  { ProfScope ps(c, 3, 0.0); launch_plan(c->stream, causal ? 3 : 2, 0, N, B, d.mask_id, 1, kv->seq_len, st->block_pos0, st->block_tokens, st->carry_tokens,
              nullptr, c->plan, scratch->logit_row_of, nullptr, nullptr, scratch->stage_row0, scratch->stage_lead, nullptr, nullptr); }
  if ((rc = forward(c, kv, N, B, scratch->k_stage, scratch->v_stage, scratch->logits_ver))) return rc;
  const KvGeom g = geom(c, kv);
  // every staged row is appended: lead = rows, accepted = 0 (the zero array stands in for n_accept and span_len)
  { ProfScope ps(c, 3, 0.0); launch_kv_append(c->stream, d.dtype, d.n_layers, N, c->rows_cap, g, kv->k_pages, kv->v_pages,
                   scratch->k_stage, scratch->v_stage, scratch->stage_row0, scratch->stage_lead, c->zeros_i32, c->zeros_i32,
                   kv->seq_len, kv->status, B, 0); }
  return check_launch("s2d2_block_complete");
}

int32_t s2d2_block_advance(s2d2_ctx* c, const s2d2_kv_view* kv, const s2d2_block_state* st, int32_t N, int32_t B,
                           uint32_t* step_dev) {
  int32_t rc;
  if ((rc = check_state(c, st, N, B)) || (rc = check_kv(c, kv))) return rc;
  launch_block_advance(c->stream, N, B, c->desc.mask_id, kv->seq_len, st->block_pos0, st->block_tokens,
                       st->carry_tokens, step_dev, kv->status);
  return check_launch("s2d2_block_advance");
}

int32_t s2d2_commit_threshold(s2d2_ctx* c, const s2d2_block_state* st, int32_t N, int32_t B,
                              const s2d2_draft_out* draft) {
  int32_t rc;
  if ((rc = check_state(c, st, N, B)) || (rc = check_draft_out(draft))) return rc;
  launch_commit_threshold(c->stream, N, B, st->block_tokens, draft->xhat, draft->unmask);
  return check_launch("s2d2_commit_threshold");
}

int32_t s2d2_route(s2d2_ctx* c, int32_t N, int32_t B, const s2d2_route_params* rp, const s2d2_draft_out* draft,
                   int32_t* hysteresis, const s2d2_route_out* out) {
  int32_t rc;
  if (!c) return fail(S2D2_EINVAL, "ctx is NULL");
  if (N < 1 || N > c->max_batch || B < 1 || B > c->max_block) return fail(S2D2_EINVAL, "N=%d or B=%d outside the limits given to s2d2_create (%d, %d)", N, B, c->max_batch, c->max_block);
  if ((rc = check_draft_out(draft))) return rc;
  if (!rp) return fail(S2D2_EINVAL, "route parameters are NULL");
  if (rp->policy < S2D2_ROUTE_MIN_SPAN || rp->policy > S2D2_ROUTE_HYSTERESIS) return fail(S2D2_EINVAL, "unknown routing policy %d", rp->policy);
  if (rp->estimator != S2D2_EST_MARGIN && rp->estimator != S2D2_EST_ENTROPY) return fail(S2D2_EINVAL, "unknown acceptance estimator %d", rp->estimator);
  if (rp->tau_span < 0) return fail(S2D2_EINVAL, "tau_span=%d is negative", rp->tau_span);
  if (rp->policy == S2D2_ROUTE_HYSTERESIS && !hysteresis) return fail(S2D2_EINVAL, "the hysteresis policy needs the state array");
  if (!out || !out->do_verify || !out->khat || !out->score || !out->unmask_fallback) return fail(S2D2_EINVAL, "route output or one of its pointers is NULL");
  { ProfScope ps(c, 3, 0.0); launch_route(c->stream, N, B, *rp, draft->span_start, draft->span_len, draft->margin, draft->entropy_n, draft->n_hi,
               draft->unmask, hysteresis, out->do_verify, out->khat, out->score, out->unmask_fallback); }
  return check_launch("s2d2_route");
}

int32_t s2d2_profile_start(s2d2_ctx* c, int32_t max_launches) {
  if (!c) return fail(S2D2_EINVAL, "ctx is NULL");
  if (max_launches < 1 || max_launches > (1 << 20)) return fail(S2D2_EINVAL, "max_launches must be in [1, 2^20]");
  if (!c->prof) { c->prof = new std::vector<s2d2_ctx::ProfRec>(); c->prof_pool = new std::vector<hipEvent_t>(); }
  while ((int32_t)c->prof_pool->size() < 2 * max_launches) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return fail(S2D2_ELAUNCH, "hipEventCreate failed");
    c->prof_pool->push_back(e);
  }
  c->prof->clear();
  c->prof_cap = max_launches;
  c->prof_on = true;
  return S2D2_OK;
}

int32_t s2d2_profile_stop(s2d2_ctx* c, s2d2_profile* out) {
  if (!c || !out) return fail(S2D2_EINVAL, "NULL argument");
  if (!c->prof_on) return fail(S2D2_EINVAL, "profiling is not on");
  c->prof_on = false;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(S2D2_ELAUNCH, "stream synchronize failed");
  for (int k = 0; k < S2D2_PROFILE_CLASSES; ++k) out[k] = s2d2_profile{0, 0.0, 0.0, 0.0, 0.0};
  for (const auto& r : *c->prof) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) { (void)hipGetLastError(); continue; }   // scope without a launch
    for (int k : {r.cls, r.sub}) {
      if (k < 0) continue;
      out[k].launches += 1;
      out[k].ms += ms;
      out[k].bytes += r.bytes;
      out[k].flops += r.flops;
      if (ms > out[k].max_ms) out[k].max_ms = ms;
    }
  }
  return S2D2_OK;
}

int32_t s2d2_status(s2d2_ctx* c) {
  if (!c) return fail(S2D2_EINVAL, "ctx is NULL");
  int32_t flag[2] = {0, 0};
  if (hipStreamSynchronize(c->stream) != hipSuccess || hipMemcpy(flag, c->dev_status, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess)
    return fail(S2D2_ELAUNCH, "could not read the device status: %s", hipGetErrorString(hipGetLastError()));
  if (flag[1]) return fail(S2D2_ELAUNCH, "a workgroup of the streaming GEMM waited in vain for its partner's share of K");
  return S2D2_OK;
}

int32_t s2d2_debug_buffer(s2d2_ctx* c, const char* name, void** ptr) {
  if (!c || !name || !ptr) return fail(S2D2_EINVAL, "NULL argument");
  const struct { const char* n; void* p; } tab[] = {{"h", c->h}, {"a", c->a}, {"q", c->qbuf}, {"o", c->obuf}, {"ffn", c->ffn},
                                                    {"kwin", c->kwin}, {"vwin", c->vwin}, {"ss", c->ss}, {"tstamp", c->ts_scratch}};
  if (!strcmp(name, "stream_ts")) { launch_stream_ts_copy(c->stream, c->ts_scratch); *ptr = c->ts_scratch; return S2D2_OK; }
  if (!strcmp(name, "tile_ts")) { launch_tile_ts_copy(c->stream, c->ts_scratch); *ptr = c->ts_scratch; return S2D2_OK; }
  if (!strcmp(name, "wide_ts")) { launch_wide_ts_copy(c->stream, c->ts_scratch); *ptr = c->ts_scratch; return S2D2_OK; }
  if (!strcmp(name, "attn_ts")) { launch_attn_ts_copy(c->stream, c->ts_scratch); *ptr = c->ts_scratch; return S2D2_OK; }
  for (const auto& t : tab)
    if (!strcmp(t.n, name)) { *ptr = t.p; return S2D2_OK; }
  return fail(S2D2_EINVAL, "unknown buffer %s", name);
}

int32_t s2d2_moe_choices(s2d2_ctx* c, int32_t rows, int32_t* out) {
  if (!c || !out) return fail(S2D2_EINVAL, "NULL argument");
  if (c->desc.n_experts == 0) return fail(S2D2_EINVAL, "not a MoE model");
  if (rows < 1 || rows > c->rows_cap) return fail(S2D2_EINVAL, "rows=%d outside [1, %d]", rows, c->rows_cap);
  launch_moe_copy_choices(c->stream, c->moe_choice, out, c->desc.n_layers, c->rows_cap * c->desc.top_k, rows * c->desc.top_k);
  return check_launch("s2d2_moe_choices");
}

int32_t s2d2_vocab_draft_stats(s2d2_ctx* c, const float* logits, int32_t rows, int32_t* xhat, float* p, float* lse,
                               float* margin, float* entropy_n) {
  if (!c) return fail(S2D2_EINVAL, "ctx is NULL");
  if (rows < 0 || rows > c->logit_cap) return fail(S2D2_EINVAL, "rows=%d outside [0, max_batch*max_block=%d]", rows, c->logit_cap);
  if (!logits || !xhat || !p || !lse || !margin || !entropy_n) return fail(S2D2_EINVAL, "NULL argument");
  if ((uintptr_t)logits & 15) return fail(S2D2_EINVAL, "logits must be 16-byte aligned");
  if (rows == 0) return S2D2_OK;
  S2D2_LAUNCH(set_i32_kernel, dim3(1), dim3(1), 0, c->stream, c->tmp_count, rows);
  launch_vocab_draft(c->stream, logits, c->desc.vocab, c->tmp_count, rows, c->vws, nullptr, nullptr, 0, xhat, p, lse,
                     margin, entropy_n, VocabSample{false, 1.0f, 0, 0, nullptr});
  return check_launch("s2d2_vocab_draft_stats");
}

int32_t s2d2_vocab_score(s2d2_ctx* c, const float* logits_ver, int32_t rows, const int32_t* token, float* q, float* lse) {
  if (!c) return fail(S2D2_EINVAL, "ctx is NULL");
  if (rows < 0 || rows > c->logit_cap) return fail(S2D2_EINVAL, "rows=%d outside [0, max_batch*max_block=%d]", rows, c->logit_cap);
  if (!logits_ver || !token || !q || !lse) return fail(S2D2_EINVAL, "NULL argument");
  if ((uintptr_t)logits_ver & 15) return fail(S2D2_EINVAL, "logits must be 16-byte aligned");
  if (rows == 0) return S2D2_OK;
  S2D2_LAUNCH(set_i32_kernel, dim3(1), dim3(1), 0, c->stream, c->tmp_count, rows);
  launch_vocab_score(c->stream, logits_ver, c->desc.vocab, c->tmp_count, rows, c->vws, nullptr, nullptr, 0, token, q, lse, 1.0f);
  return check_launch("s2d2_vocab_score");
}

}  // extern "C"
