// Window construction and per-sequence state kernels (integer work only).
//
// plan_kernel builds, on the device and without host involvement, the packed list of window
// rows of a draft forward (block positions not yet cached, Eq. 4 visibility) or of a verifier
// forward (the 2L window of Eq. 3 with uncached committed tokens riding in front as causal
// rows).  kv_append / block_advance / commit_threshold update the per-sequence state
// (Algorithm 1 append and new block; Algorithm 2 commit).
#include "s2d2_internal.h"
#include "../../include/s2d2.h"

namespace s2d2 {

// The token arrays live on the device and cannot be checked by the host: an id outside the vocabulary (a caller's
// mistake, or the proposal of a logit row without a single comparable value) becomes [MASK] instead of an
// embedding row outside the table.
__device__ __forceinline__ int in_vocab(int tok, int vocab, int mask_id) { return (unsigned)tok < (unsigned)vocab ? tok : mask_id; }

__global__ __launch_bounds__(1024) void plan_kernel(
    int verify, int shifted, int N, int B, int mask_id, int ar_mask, const int32_t* __restrict__ seq_len,
    const int32_t* __restrict__ pos0, const int32_t* __restrict__ block,
    const int32_t* __restrict__ carry, const int32_t* __restrict__ xhat, Plan p,
    int32_t* __restrict__ logit_row_of, int32_t* __restrict__ span_start,
    int32_t* __restrict__ span_len, int32_t* __restrict__ stage_row0, int32_t* __restrict__ stage_lead,
    const int32_t* __restrict__ active, int32_t* __restrict__ status, float* __restrict__ clear_a,
    float* __restrict__ clear_b) {
  __shared__ int32_t s_rows[1024];
  __shared__ int32_t s_lrows[1024];
  const int n = threadIdx.x;
  int S = 0, c = 0, nc = 0, j = B, L = 0, n_masked = 0, rows = 0, lrows = 0, lead = 0, bad = 0;
  if (n < N) {
    S = seq_len[n];
    const int P0 = pos0[n];
    c = max(0, min(B, S - P0));
    nc = max(0, min(B, P0 - S));
    const int32_t* blk = block + (size_t)n * B;
    for (int i = 0; i < B; ++i) {
      const bool m = blk[i] == mask_id;
      n_masked += m;
      if (m && j == B) j = i;
    }
    while (j + L < B && blk[j + L] == mask_id) ++L;
    c = min(c, j);
    lead = nc + (j - c);
    if (verify == 1 && active && active[n] == 0) { L = 0; lead = 0; }   // routed to the fallback: no verifier window
    // right-shifted model: the row in front of the first [MASK] scores it and has to be a window row
    if (shifted && verify < 2 && L > 0 && lead == 0) {
      if (status) status[n] = S2D2_EINVAL;
      if (verify) L = 0;
      bad = 1;
    }
    if (verify >= 2) {            // block completion: all uncached tokens of a finished block, no logits
      rows = n_masked == 0 ? nc + (B - c) : 0;
      if (verify == 3 && rows <= B) rows = 0;   // causal variant: only what the carry list (capacity B) cannot take
      lead = rows;
      lrows = 0;
    } else if (verify) { rows = shifted ? lead + max(L - 1, 0) : lead + 2 * L; lrows = L; }
    else        { rows = nc + (B - c); lrows = bad ? 0 : n_masked; }
  }
  s_rows[n] = rows;
  s_lrows[n] = lrows;
  __syncthreads();
  // inclusive Hillis-Steele scan over the 1024 slots
  for (int off = 1; off < 1024; off <<= 1) {
    int a = 0, b = 0;
    if (n >= off) { a = s_rows[n - off]; b = s_lrows[n - off]; }
    __syncthreads();
    s_rows[n] += a;
    s_lrows[n] += b;
    __syncthreads();
  }
  if (n == 1023) { p.counts[0] = s_rows[1023]; p.counts[1] = s_lrows[1023]; }
  if (n >= N) return;
  const int row0 = s_rows[n] - rows;
  int k = s_lrows[n] - lrows;
  p.seq_row0[n] = row0;
  p.seq_rows[n] = rows;
  p.seq_lead[n] = lead;
  p.seq_j[n] = j;
  p.seq_L[n] = L;
  const int32_t* blk = block + (size_t)n * B;
  const int32_t* car = carry + (size_t)n * B;
  if (!verify) {
    span_start[n] = j;
    span_len[n] = bad ? 0 : L;   // a skipped sequence has nothing to verify, accept or append
    for (int i = 0; i < B; ++i) logit_row_of[(size_t)n * B + i] = -1;
    for (int t = 0; t < rows; ++t) {
      const int r = row0 + t;
      int tok, hi;
      if (t < nc) {                       // carried token of a finished block: causal
        tok = car[t];
        hi = r + 1;
      } else {
        const int i = c + (t - nc);
        tok = blk[i];
        hi = (i < j && ar_mask) ? r + 1 : row0 + rows;   // Eq. 4: committed prefix causal, rest sees all
        if (tok == mask_id && !bad) {
          p.logit_src[k] = r - shifted;   // right-shifted model: the row in front (t >= 1 here: lead >= 1)
          p.logit_seq[k] = n;
          p.logit_idx[k] = i;
          logit_row_of[(size_t)n * B + i] = k;
          ++k;
        }
      }
      p.row_token[r] = in_vocab(tok, p.vocab, mask_id);
      p.row_pos[r] = S + t;
      p.row_seq[r] = n;
      p.row_lo[r] = row0;
      p.row_hi[r] = hi;
    }
  } else if (verify >= 2) {
    // Alg. 1 after the block sampler: carried tokens stay causal, the block's rows attend to the whole window
    // (block-diffusion attention; verify == 3: every row causal, Section 4.2); every row is staged for the cache
    stage_row0[n] = row0;
    stage_lead[n] = rows;
    for (int t = 0; t < rows; ++t) {
      const int r = row0 + t;
      p.row_token[r] = in_vocab(t < nc ? car[t] : blk[c + (t - nc)], p.vocab, mask_id);
      p.row_pos[r] = S + t;
      p.row_seq[r] = n;
      p.row_lo[r] = row0;
      p.row_hi[r] = (t < nc || verify == 3) ? r + 1 : row0 + rows;
    }
  } else {
    stage_row0[n] = row0;
    stage_lead[n] = lead;
    for (int i = 0; i < B; ++i) logit_row_of[(size_t)n * B + i] = -1;
    // per-position outputs of the verifier (q, lse) start at zero; the vocabulary pass fills the planned positions
    if (clear_a)
      for (int i = 0; i < B; ++i) { clear_a[(size_t)n * B + i] = 0.f; clear_b[(size_t)n * B + i] = 0.f; }
    const int32_t* xh = xhat + (size_t)n * B;
    const int n_drafted = shifted ? max(L - 1, 0) : L;   // a right-shifted window has no row for the last drafted token
    for (int t = 0; t < lead + n_drafted; ++t) {  // causal half: carry, pending committed, drafted C_t
      const int r = row0 + t;
      int tok;
      if (t < nc) tok = car[t];
      else if (t < lead) tok = blk[c + (t - nc)];
      else tok = xh[j + (t - lead)];
      p.row_token[r] = in_vocab(tok, p.vocab, mask_id);
      p.row_pos[r] = S + t;
      p.row_seq[r] = n;
      p.row_lo[r] = row0;
      p.row_hi[r] = r + 1;
    }
    for (int q = 0; q < L && shifted; ++q) {   // right-shifted: row of position i-1 scores the drafted token at i
      p.logit_src[k] = row0 + lead - 1 + q;
      p.logit_seq[k] = n;
      p.logit_idx[k] = j + q;
      logit_row_of[(size_t)n * B + j + q] = k;
      ++k;
    }
    for (int q = 0; q < L && !shifted; ++q) {   // [MASK] copies: see causal rows strictly left, and themselves
      const int r = row0 + lead + L + q;
      p.row_token[r] = mask_id;
      p.row_pos[r] = S + lead + q;
      p.row_seq[r] = n;
      p.row_lo[r] = row0;
      p.row_hi[r] = row0 + lead + q;
      p.logit_src[k] = r;
      p.logit_seq[k] = n;
      p.logit_idx[k] = j + q;
      logit_row_of[(size_t)n * B + j + q] = k;
      ++k;
    }
  }
}

void launch_plan(hipStream_t st, int verify, int shifted, int N, int B, int mask_id, int ar_mask,
                 const int32_t* seq_len, const int32_t* pos0, const int32_t* block,
                 const int32_t* carry, const int32_t* xhat, const Plan& p, int32_t* logit_row_of,
                 int32_t* span_start, int32_t* span_len, int32_t* stage_row0, int32_t* stage_lead,
                 const int32_t* active, int32_t* status, float* clear_a, float* clear_b) {
  S2D2_LAUNCH(plan_kernel, dim3(1), dim3(1024), 0, st, verify, shifted, N, B, mask_id, ar_mask,
                     seq_len, pos0, block, carry, xhat, p, logit_row_of, span_start, span_len,
                     stage_row0, stage_lead, active, status, clear_a, clear_b);
}

// ---------------------------------------------------------------------------------------------
// Cache append: copy staged K/V rows [0, lead + n_accept) of each sequence to its next logical
// positions.  One workgroup per (sequence, staged row, layer); 16-byte copies.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void kv_append_copy_kernel(
    int elt_bytes, int per_seq, int rows_cap, KvGeom g, uint8_t* __restrict__ k_pages,
    uint8_t* __restrict__ v_pages, const uint8_t* __restrict__ k_stage, const uint8_t* __restrict__ v_stage,
    const int32_t* __restrict__ stage_row0, const int32_t* __restrict__ stage_lead,
    const int32_t* __restrict__ n_accept, const int32_t* __restrict__ span_len, int hold_back) {
  const int n = blockIdx.x / per_seq, t = blockIdx.x % per_seq, l = blockIdx.y;
  const int acc = max(0, min(n_accept[n], span_len[n] - hold_back));   // hold_back: no staged row for the last drafted token
  const int rows = stage_lead[n] + acc;
  if (t >= rows) return;
  const int S = g.seq_len[n];
  const int cap = g.max_pages_per_seq * g.page_size;
  if (S + rows > cap) return;  // whole sequence skipped; the update kernel flags it
  const int s = S + t;
  const int page = g.page_table[(size_t)n * g.max_pages_per_seq + s / g.page_size];
  if (page < 0 || page >= g.n_pages) return;
  const int slot = s % g.page_size;
  const size_t head_bytes = (size_t)g.head_dim * elt_bytes;
  const size_t src = ((size_t)l * rows_cap + (stage_row0[n] + t)) * g.n_kv_heads * head_bytes;
  const size_t layer_off = (size_t)l * g.n_pages * g.n_kv_heads * g.page_size * head_bytes;
  const int vec_per_head = (int)(head_bytes / 16);
  for (int v = threadIdx.x; v < g.n_kv_heads * vec_per_head; v += blockDim.x) {
    const int h = v / vec_per_head, e = v % vec_per_head;
    const size_t dst = layer_off + (((size_t)page * g.n_kv_heads + h) * g.page_size + slot) * head_bytes + (size_t)e * 16;
    *(uint4*)(k_pages + dst) = *(const uint4*)(k_stage + src + (size_t)h * head_bytes + (size_t)e * 16);
  }
  // V is cached key-minor: [page, Hkv, D, page_size]
  for (int v = threadIdx.x; v < g.n_kv_heads * g.head_dim; v += blockDim.x) {
    const int h = v / g.head_dim, d = v % g.head_dim;
    const size_t dst = layer_off + ((((size_t)page * g.n_kv_heads + h) * g.head_dim + d) * g.page_size + slot) * elt_bytes;
    const size_t so = src + (size_t)v * elt_bytes;
    if (elt_bytes == 2) *(uint16_t*)(v_pages + dst) = *(const uint16_t*)(v_stage + so);
    else *(uint32_t*)(v_pages + dst) = *(const uint32_t*)(v_stage + so);
  }
}

__global__ void kv_append_commit_kernel(int N, KvGeom g, const int32_t* __restrict__ stage_lead,
                                        const int32_t* __restrict__ n_accept,
                                        const int32_t* __restrict__ span_len, int32_t* __restrict__ seq_len,
                                        int32_t* __restrict__ status, int hold_back) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  const int acc = max(0, min(n_accept[n], span_len[n] - hold_back));
  const int rows = stage_lead[n] + acc;
  const int S = seq_len[n];
  if (S + rows > g.max_pages_per_seq * g.page_size) {
    if (status) status[n] = S2D2_ENOSPC;
    return;
  }
  seq_len[n] = S + rows;
}

void launch_kv_append(hipStream_t st, int dtype, int n_layers, int N, int rows_cap, const KvGeom& g,
                      void* k_pages, void* v_pages, const void* k_stage, const void* v_stage,
                      const int32_t* stage_row0, const int32_t* stage_lead, const int32_t* span_len,
                      const int32_t* n_accept, int32_t* seq_len, int32_t* status, int B, int hold_back) {
  const int elt = dtype == S2D2_BF16 ? 2 : 4;
  const int per_seq = 2 * B;  // upper bound of staged causal rows per sequence (carry + block)
  S2D2_LAUNCH(kv_append_copy_kernel, dim3(N * per_seq, n_layers), dim3(256), 0, st, elt, per_seq,
                     rows_cap, g, (uint8_t*)k_pages, (uint8_t*)v_pages, (const uint8_t*)k_stage,
                     (const uint8_t*)v_stage, stage_row0, stage_lead, n_accept, span_len, hold_back);
  S2D2_LAUNCH(kv_append_commit_kernel, dim3((N + 255) / 256), dim3(256), 0, st, N, g, stage_lead,
                     n_accept, span_len, seq_len, status, hold_back);
}

// ---------------------------------------------------------------------------------------------
// Alg. 1: replace a block that holds no [MASK] by a fresh [MASK]^B block right after it.
// Uncached committed tokens of the finished block move to the carry list (capacity B); if they
// would not fit, the block is left as it is and the sequence's status word says so (the caller
// caches them first: s2d2_block_complete).
// ---------------------------------------------------------------------------------------------
__global__ void block_advance_kernel(int N, int B, int mask_id, const int32_t* __restrict__ seq_len,
                                     int32_t* __restrict__ pos0, int32_t* __restrict__ block,
                                     int32_t* __restrict__ carry, uint32_t* step_dev, int32_t* __restrict__ status) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n == 0 && step_dev) *step_dev += 1u;
  if (n >= N) return;
  int32_t* blk = block + (size_t)n * B;
  int32_t* car = carry + (size_t)n * B;
  for (int i = 0; i < B; ++i)
    if (blk[i] == mask_id) return;
  const int S = seq_len[n], P0 = pos0[n];
  const int c = max(0, min(B, S - P0)), nc = max(0, min(B, P0 - S));
  if (nc + (B - c) > B) {
    if (status) status[n] = S2D2_ENOSPC;
    return;
  }
  for (int i = c; i < B; ++i) car[nc + (i - c)] = blk[i];
  for (int i = 0; i < B; ++i) blk[i] = mask_id;
  pos0[n] = P0 + B;
}

void launch_block_advance(hipStream_t st, int N, int B, int mask_id, const int32_t* seq_len,
                          int32_t* pos0, int32_t* block, int32_t* carry, uint32_t* step_dev, int32_t* status) {
  S2D2_LAUNCH(block_advance_kernel, dim3((N + 255) / 256), dim3(256), 0, st, N, B, mask_id, seq_len,
                     pos0, block, carry, step_dev, status);
}

__global__ void commit_threshold_kernel(int N, int B, int32_t* __restrict__ block,
                                        const int32_t* __restrict__ xhat, const uint64_t* __restrict__ unmask) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= N * B) return;
  const int n = idx / B, i = idx % B;
  if ((unmask[n] >> i) & 1ull) block[idx] = xhat[idx];
}

void launch_commit_threshold(hipStream_t st, int N, int B, int32_t* block, const int32_t* xhat,
                             const uint64_t* unmask) {
  S2D2_LAUNCH(commit_threshold_kernel, dim3((N * B + 255) / 256), dim3(256), 0, st, N, B, block, xhat,
                     unmask);
}

// ---------------------------------------------------------------------------------------------
// Verification routing (Section 4.3): one thread per sequence.  K = sum_k prod_{i<=k} alpha_i over C_t,
// score, policy decision, hysteresis state update.
// ---------------------------------------------------------------------------------------------
__global__ void route_kernel(int N, int B, s2d2_route_params rp, const int32_t* __restrict__ span_start,
                             const int32_t* __restrict__ span_len, const float* __restrict__ margin,
                             const float* __restrict__ entropy_n, const int32_t* __restrict__ n_hi,
                             const uint64_t* __restrict__ unmask, int32_t* __restrict__ hysteresis,
                             int32_t* __restrict__ do_verify, float* __restrict__ khat, float* __restrict__ score,
                             uint64_t* __restrict__ unmask_fallback) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  const int j = span_start[n], L = max(0, min(span_len[n], B - j));
  float prod = 1.f, k = 0.f;
  for (int i = 0; i < L; ++i) {
    const int o = n * B + j + i;
    const float a = rp.estimator == S2D2_EST_MARGIN ? (margin[o] >= rp.tau_margin ? 1.f : 0.f)
                                                    : expf(-rp.beta * entropy_n[o]);
    prod *= a;
    k += prod;
  }
  const float s = rp.dynamic ? k - rp.c * (float)n_hi[n] : k - rp.c;
  bool dec;
  if (rp.policy == S2D2_ROUTE_MIN_SPAN) {
    dec = L >= rp.tau_span;
  } else if (rp.policy == S2D2_ROUTE_SCORE) {
    dec = s >= rp.tau_score;
  } else {
    int h = hysteresis[n] != 0;
    if (L > 0) {   // a block without a masked span leaves the state as it is
      if (h && s < rp.tau_off) h = 0;
      else if (!h && s >= rp.tau_on) h = 1;
      hysteresis[n] = h;
    }
    dec = h != 0;
  }
  dec = dec && L > 0;
  do_verify[n] = dec ? 1 : 0;
  khat[n] = k;
  score[n] = s;
  unmask_fallback[n] = dec ? 0ull : unmask[n];
}

void launch_route(hipStream_t st, int N, int B, const s2d2_route_params& rp, const int32_t* span_start,
                  const int32_t* span_len, const float* margin, const float* entropy_n, const int32_t* n_hi,
                  const uint64_t* unmask, int32_t* hysteresis, int32_t* do_verify, float* khat, float* score,
                  uint64_t* unmask_fallback) {
  S2D2_LAUNCH(route_kernel, dim3((N + 255) / 256), dim3(256), 0, st, N, B, rp, span_start, span_len, margin,
              entropy_n, n_hi, unmask, hysteresis, do_verify, khat, score, unmask_fallback);
}

}  // namespace s2d2
