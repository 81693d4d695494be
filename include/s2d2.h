/*
 * s2d2.h - C ABI of the S2D2 draft + verify + accept + cache-append step for MI355X (gfx950).
 *
 * The library runs ONE decoding step of self-speculative block-diffusion decoding
 * (paper: Section 4.1-4.2, Algorithm 3) on a batch of independent sequences:
 *
 *   s2d2_draft        draft forward under block-diffusion attention (Eq. 4), SampleFromLogits,
 *                     masked set M_t, first contiguous masked span C_t, threshold set (Alg. 2)
 *   s2d2_verify       verifier forward under block-size-1 masking (the 2L window of Eq. 3),
 *                     ScoreFromLogits
 *   s2d2_accept       left-to-right speculative acceptance, residual resampling, commit
 *   s2d2_kv_append    append K/V of the accepted prefix to the paged cache (Alg. 1 append,
 *                     with the causal "AR caching" of Section 4.2)
 *   s2d2_block_advance  start a fresh [MASK]^B block when the current one is complete (Alg. 1)
 *   s2d2_commit_threshold  the confidence-threshold commit (Alg. 2 / else-branch of Alg. 3)
 *
 * Conventions
 *   - Every pointer marked "device" is caller-owned device memory; "host" is host memory.
 *     The library allocates no device memory: the caller provides a workspace whose size
 *     s2d2_workspace_bytes() reports.  Host memory for the context is malloc'ed by
 *     s2d2_create and released by s2d2_destroy.
 *   - Every call only enqueues kernels on the context's stream and returns; it never
 *     synchronises and never reads device results.  Outputs are valid once the caller has
 *     synchronised that stream.  No memset / memcpy nodes are issued, so a sequence of calls
 *     can be captured into a HIP graph.
 *   - Arguments are validated on the host before anything is launched.  Return value: 0 or a
 *     negative S2D2_E* code; s2d2_last_error() gives a human-readable reason.
 *   - Conditions that only the device can see (a sequence that runs out of pages) set the
 *     per-sequence `status` word and skip the write; they never fault.
 *   - Same inputs and same (seed, step) give bit-identical outputs: no float atomics.
 *
 * Per-sequence decoding state (device, read and updated by the calls):
 *   seq_len[n]        tokens whose K/V are in the cache (positions 0 .. seq_len-1)
 *   block_pos0[n]     absolute position of block index 0
 *   block_tokens[n,B] committed token id, or mask_id where the position is still [MASK]
 *   carry_tokens[n,B] committed tokens of earlier blocks that are not cached yet; they occupy
 *                     positions seq_len .. block_pos0-1 (count = block_pos0 - seq_len if > 0).
 *   If seq_len >= block_pos0, the first seq_len - block_pos0 block positions are cached.
 *   Token ids are device data the host cannot check: a forward reads an id outside [0, vocab) as mask_id
 *   (never as an embedding row outside the table), and a logit row without one comparable value (all NaN)
 *   proposes token 0.
 */
#ifndef S2D2_H
#define S2D2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define S2D2_OK        0
#define S2D2_EINVAL   -1   /* null / misaligned / out-of-range argument */
#define S2D2_ENOSPC   -2   /* workspace or page table too small */
#define S2D2_EARCH    -3   /* current device is not gfx950 */
#define S2D2_ELAUNCH  -4   /* HIP runtime error while enqueueing */

#define S2D2_F32   0
#define S2D2_BF16  1

#define S2D2_GREEDY 0      /* x_hat = arg-max, p = softmax(logits)[x_hat] */
#define S2D2_SAMPLE 1      /* x_hat ~ softmax(logits / temperature) by inverse CDF in ascending token order (stream 2
                            * uniform); p, q, margin, entropy and the residual are then all taken at that temperature */

#define S2D2_MAX_BLOCK 64  /* B <= 64: per-sequence sets are returned as 64-bit masks */

typedef struct s2d2_ctx s2d2_ctx;

/* Decoder shape.  Pre-norm blocks: RMSNorm, GQA attention with half-split RoPE, SwiGLU FFN
 * (n_experts == 0) or softmax-top-k MoE of SwiGLU experts (n_experts > 0: bf16 only, n_experts <= 256,
 * top_k <= 64; router = softmax over all experts, top-k by value with ties to the lower index, weights
 * renormalised to sum 1, no shared expert, no capacity limit).
 * Limits (S2D2_EINVAL beyond them): n_layers <= 4096, 32 <= d_model <= 65536, n_q_heads <= 1024, head_dim in
 * {32, 64, 128, 256}, d_ffn and d_expert <= 1048576, vocab <= 2097152. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t n_experts, top_k, d_expert;   /* all 0 for a dense model */
  int32_t dtype;                        /* S2D2_F32 or S2D2_BF16: weights, KV cache, activations */
  int32_t mask_id;                      /* token id of [MASK] */
  int32_t act_planes;                   /* bf16 models with packed weights: how the inputs of the GEMMs are carried.
                                           3 (also chosen by 0, the default): as IEEE half values, 11 significant
                                           bits, against a half copy of the weights made when the packed buffer is
                                           filled (bf16 -> half is exact for |w| >= 2^-17, absolute error <= 2^-25
                                           below), on the f16 MFMA, whose rate equals the bf16 one; needs activations
                                           within the half range (|x| < 65504);
                                           2: as a high- and a low-order bf16 plane, 16 significant bits, every bf16
                                           weight operand multiplied with both (twice the matrix instructions);
                                           1: one bf16 plane, 8 significant bits (36-layer models leave the 2e-2 logit
                                           tolerance against an fp64 reference with it).
                                           Queries, keys, values and the KV cache are bf16 in every mode. */
  int32_t right_shifted;                /* 1: the model's output at position i-1 is the distribution of token i
                                           (Section 4.2, right-shifted models).  s2d2_draft then reads the logits of a
                                           masked block position from the window row in front of it, s2d2_verify runs
                                           span_len plain causal rows (the uncached committed tokens left of C_t and the
                                           first span_len - 1 drafted tokens, no [MASK] copies) and s2d2_kv_append never
                                           caches the last drafted token.  Precondition, kept by these calls once it
                                           holds: the committed token in front of the first [MASK] is not cached yet
                                           (after a prompt of S tokens: seq_len = S - 1, block_pos0 = S, carry_tokens[0] =
                                           last prompt token).  A sequence that violates it gets status S2D2_EINVAL and
                                           is skipped.  s2d2_block_complete is refused.  0: logits of the [MASK] rows. */
  float rope_theta, rms_eps;
} s2d2_model_desc;

/* Device pointers of one layer.  "out, in" layouts, input dimension contiguous, in `dtype`;
 * norm gains are fp32 [d_model].
 *   wqkv  [(Hq + 2 Hkv) * D, d]   rows: query heads, key heads, value heads
 *   wo    [d, Hq * D]
 *   wgu   [2, F, d] ([0] gate, [1] up)      wdown [d, F]            (dense)
 *   router [E, d]   e_wgu [E, 2, Fe, d]     e_wdown [E, d, Fe]      (MoE) */
typedef struct {
  const float* norm1;
  const void* wqkv;
  const void* wo;
  const float* norm2;
  const void* wgu;
  const void* wdown;
  const void* router;
  const void* e_wgu;
  const void* e_wdown;
} s2d2_layer_weights;

typedef struct {
  const void* embed;                  /* device [V, d] */
  const void* unembed;                /* device [V, d] */
  const float* norm_f;                /* device [d] */
  const s2d2_layer_weights* layers;   /* HOST array [n_layers] of device pointers (copied) */
} s2d2_weights;

/* Paged prefix cache, shared page table for all layers.
 *   k_pages   device [n_layers, n_pages, Hkv, page_size, D] in `dtype`, keys stored after RoPE
 *   v_pages   device [n_layers, n_pages, Hkv, D, page_size] in `dtype`: values are stored key-minor
 *             (transposed inside a page) so that the P*V contraction index is contiguous for MFMA
 *             Logical position s of sequence n lives in physical page page_table[n, s / page_size],
 *             slot s % page_size.  page_size % 8 == 0 selects the MFMA attention kernel for bf16
 *             models with head_dim 128; other shapes run a plain fp32 kernel.
 *   status            device [N], set to S2D2_ENOSPC by s2d2_kv_append for a sequence whose
 *                     append would pass max_pages_per_seq * page_size (nothing is written for
 *                     it), else left unchanged.  May be NULL. */
typedef struct {
  void* k_pages;
  void* v_pages;
  const int32_t* page_table;   /* device [N, max_pages_per_seq] */
  int32_t* seq_len;            /* device [N], advanced by s2d2_kv_append */
  int32_t* status;             /* device [N] or NULL */
  int32_t n_pages, page_size, max_pages_per_seq;
} s2d2_kv_view;

typedef struct {
  int32_t* block_tokens;   /* device [N, B] */
  int32_t* block_pos0;     /* device [N] */
  int32_t* carry_tokens;   /* device [N, B] */
} s2d2_block_state;

/* Sampling / acceptance parameters (host, by value).
 *   Uniforms are Philox-4x32-10 draws: key = seed, counter = (step, n, block index, stream)
 *   with stream 0 = accept test, 1 = residual draw, 2 = draft sampling;
 *   u = (top 23 bits + 0.5) / 2^23.  If step_dev is non-NULL the step word is
 *   step + *step_dev, and s2d2_block_advance increments *step_dev (graph replay). */
typedef struct {
  float tau;            /* confidence threshold of Alg. 2 */
  float temperature;    /* used in S2D2_SAMPLE mode only */
  float gamma;          /* ratio tempering exponent, 1 = off */
  uint64_t seed;
  uint32_t step;
  int32_t mode;         /* S2D2_GREEDY | S2D2_SAMPLE */
  int32_t ar_mask;      /* 1: Eq. 4 (committed in-block prefix causal); 0: block fully bidirectional */
  int32_t resample;     /* 1: residual resampling at the first rejection; 0: reject only */
  uint32_t* step_dev;   /* device, optional */
  const int32_t* active; /* device [N] or NULL: sequences with active[n] == 0 are skipped by s2d2_verify (no window
                          * rows, nothing staged), s2d2_accept (n_accept = n_commit = 0) and hence s2d2_kv_append;
                          * NULL = all sequences.  s2d2_route writes such a mask (routing of Section 4.3). */
} s2d2_params;

/* Outputs of s2d2_draft (all device, caller-owned).  Per-position arrays are indexed
 * [n, block index]; entries of committed positions are x_hat = -1, others 0.
 *   logits        [N*B, V] fp32, compacted: row logit_row_of[n,i] holds the draft logits of
 *                 masked block position i of sequence n (-1 if that position is committed)
 *   unmask        bit i set iff i is in the threshold set {i in M_t: p_i > tau} U {argmax p}
 *   n_hi          |{i in M_t : p_i > tau}|
 *   span_start/len  C_t = first maximal run of [MASK] (len 0 if the block has none) */
typedef struct {
  float* logits;
  int32_t* logit_row_of;
  int32_t* xhat;
  float* p;
  float* lse;
  float* margin;       /* top-1 minus top-2 probability */
  float* entropy_n;    /* entropy / ln V */
  uint64_t* unmask;
  int32_t* n_hi;
  int32_t* span_start;
  int32_t* span_len;
} s2d2_draft_out;

/* Outputs of s2d2_verify (device, caller-owned).
 *   logits_ver    [N*B, V] fp32, compacted like the draft's (rows exist for C_t only)
 *   q, lse_ver    [N, B]: verifier probability of x_hat_i and log-normaliser, for i in C_t
 *   k_stage, v_stage  [n_layers, rows_cap, Hkv, D] in `dtype`, rows_cap = 3*max_batch*max_block
 *                 (s2d2_stage_rows): K (after RoPE) and V of every window row.  The rows of
 *                 sequence n start at stage_row0[n]; its first stage_lead[n] rows are the
 *                 uncached committed tokens left of C_t, the next span_len[n] rows the drafted
 *                 tokens; all of these were computed under a causal mask. */
typedef struct {
  float* logits_ver;
  int32_t* logit_row_of;
  float* q;
  float* lse_ver;
  void* k_stage;
  void* v_stage;
  int32_t* stage_row0;
  int32_t* stage_lead;
} s2d2_verify_out;

/* Outputs of s2d2_accept (device, caller-owned, [N] unless noted).
 *   n_accept      drafted tokens of C_t that passed before the first failure
 *   n_commit      n_accept + 1 if a rejection happened and resample is on
 *   resampled     residual token committed at the first rejected position, or -1
 *   u_used        [N, B] the accept uniform of each position of C_t (0 elsewhere) */
typedef struct {
  int32_t* n_accept;
  int32_t* n_commit;
  int32_t* resampled;
  float* u_used;
} s2d2_accept_out;

const char* s2d2_last_error(void);
const char* s2d2_version(void);

/* Rows of the K/V staging buffers for these limits. */
int64_t s2d2_stage_rows(int32_t max_batch, int32_t max_block);

/* Bytes of device workspace needed for these limits; negative S2D2_E* on a bad description. */
int64_t s2d2_workspace_bytes(const s2d2_model_desc* desc, int32_t max_batch, int32_t max_block);

/* Bytes of the packed copy of the projection weights that the MFMA GEMMs read (bf16 models; 0 for
 * fp32 models).  MoE models require it.  The library does not allocate it: the caller passes a device buffer
 * of this size to s2d2_create. */
int64_t s2d2_packed_bytes(const s2d2_model_desc* desc);

/* Bind weights, limits, stream (a hipStream_t, may be NULL for the default stream) and
 * workspace (device, 256-byte aligned).  `packed` (device, 256-byte aligned, s2d2_packed_bytes()
 * or NULL): if given, s2d2_create enqueues kernels that copy wqkv, wo, wgu, wdown and unembed
 * into it in MFMA tile order, and every forward reads that copy with the fused streaming GEMM;
 * the canonical copies of those five tensors may be released once the stream has run.  With
 * packed == NULL (and always for fp32 models) the canonical layouts are read by the plain
 * kernels.  embed and the norm gains stay caller-owned and must outlive ctx. */
int32_t s2d2_create(const s2d2_model_desc* desc, const s2d2_weights* weights, int32_t max_batch,
                    int32_t max_block, void* stream, void* workspace, size_t workspace_bytes,
                    void* packed, size_t packed_bytes, s2d2_ctx** out);
int32_t s2d2_destroy(s2d2_ctx* ctx);
int32_t s2d2_set_stream(s2d2_ctx* ctx, void* stream);

/* Alg. 3 draft forward, SampleFromLogits, M_t, C_t, threshold set.  N sequences, block size B. */
int32_t s2d2_draft(s2d2_ctx* ctx, const s2d2_kv_view* kv, const s2d2_block_state* st, int32_t N,
                   int32_t B, const s2d2_params* prm, const s2d2_draft_out* out);

/* Alg. 3 verifier forward on [x_hat_{C_t}, MASK^L] with the mask of Eq. 3, ScoreFromLogits. */
int32_t s2d2_verify(s2d2_ctx* ctx, const s2d2_kv_view* kv, const s2d2_block_state* st, int32_t N,
                    int32_t B, const s2d2_params* prm, const s2d2_draft_out* draft,
                    const s2d2_verify_out* out);

/* Alg. 3 accept loop + residual resample; writes committed tokens into st->block_tokens. */
int32_t s2d2_accept(s2d2_ctx* ctx, const s2d2_block_state* st, int32_t N, int32_t B,
                    const s2d2_params* prm, const s2d2_draft_out* draft,
                    const s2d2_verify_out* ver, const s2d2_accept_out* out);

/* s2d2_accept for callers that cannot allocate device memory or carry a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and results as s2d2_accept (bit for
 * bit), but no context and no workspace: the scratch of the residual draw (tile sums that the workgroups of a
 * sequence hand to each other, 4 bytes per 256 vocabulary entries and sequence, and one arrival counter per
 * sequence) lives in a device array inside the library, 512.5 KB on every GPU the library runs on, held until the
 * process ends.  Limits: N <= 128, vocab <= 262144 (2^18), B <= S2D2_MAX_BLOCK; beyond them the call returns
 * S2D2_ENOSPC and launches nothing.  `stream` is a hipStream_t (NULL: the default stream), `vocab` the width of
 * the logit rows; st->block_pos0 and st->carry_tokens are not read.  The call enqueues two kernels (a fill that
 * zeroes the arrival counters, then the accept kernel) and calls no hipMalloc, hipFree or other allocating routine;
 * the array's device address is looked up once per device (at s2d2_create, else on the first call on that device,
 * which must be current).  All calls on one GPU share the array: calls that overlap on one GPU (two streams, two
 * threads) race; calls on one stream, or otherwise ordered, are safe. */
int32_t s2d2_accept_static(void* stream, int32_t vocab, const s2d2_block_state* st, int32_t N, int32_t B,
                           const s2d2_params* prm, const s2d2_draft_out* draft, const s2d2_verify_out* ver,
                           const s2d2_accept_out* out);

/* Append the staged K/V of the leading committed rows and of C_t[0 : n_accept) to the cache
 * and advance seq_len (Alg. 1 append; Section 4.2 causal caching makes these rows final). */
int32_t s2d2_kv_append(s2d2_ctx* ctx, const s2d2_kv_view* kv, int32_t N, int32_t B,
                       const s2d2_draft_out* draft, const s2d2_verify_out* ver,
                       const int32_t* n_accept /* device [N] */);

/* Alg. 1: a block without [MASK] is replaced by a fresh [MASK]^B block at block_pos0 + B; its
 * uncached committed tokens move to carry_tokens (capacity B).  A finished block whose uncached tokens, together
 * with the tokens already carried, exceed that capacity is left as it is and kv->status[n] is set to S2D2_ENOSPC:
 * cache them first with s2d2_block_complete(..., causal = 1).  Increments *step_dev if given. */
int32_t s2d2_block_advance(s2d2_ctx* ctx, const s2d2_kv_view* kv, const s2d2_block_state* st,
                           int32_t N, int32_t B, uint32_t* step_dev /* device or NULL */);

/* Alg. 1 after the block sampler: the cache update of a finished block, one forward over its tokens that are not
 * cached yet (and over the carried tokens of earlier blocks, which stay causal) and append of their K/V; seq_len
 * advances by the rows appended, kv->status reports S2D2_ENOSPC as in s2d2_kv_append.  Sequences whose block still
 * holds a [MASK] are left alone.
 *   causal = 0  for decoding that does not append inside a block: every finished block; the block's rows attend to
 *               the whole block (block-diffusion attention).
 *   causal = 1  for decoding that appends causally (Section 4.2): every row sees only the rows left of it, so the
 *               appended K/V are those of a causal prefill; applied only to the sequences whose finished block the
 *               carry list cannot take (carried + uncached tokens > B), i.e. blocks that were finished without a
 *               verifier forward caching them.  The others keep riding in carry_tokens.
 * `scratch` supplies the staging buffers (a verify output of the same limits; its contents are overwritten).  Call
 * s2d2_block_advance afterwards. */
int32_t s2d2_block_complete(s2d2_ctx* ctx, const s2d2_kv_view* kv, const s2d2_block_state* st, int32_t N, int32_t B,
                            const s2d2_verify_out* scratch, int32_t causal);

/* Alg. 2 commit: x^b_i <- x_hat_i for every i in the draft's threshold set. */
int32_t s2d2_commit_threshold(s2d2_ctx* ctx, const s2d2_block_state* st, int32_t N, int32_t B,
                              const s2d2_draft_out* draft);

/* Verification routing (Section 4.3, Eq. 5; algorithm DoVerify): from the draft's statistics over C_t of every
 * sequence, the expected accepted prefix length K = sum_k prod_{i<=k} alpha_i with alpha_i = 1[margin_i >=
 * tau_margin] (S2D2_EST_MARGIN) or exp(-beta * entropy_n_i) (S2D2_EST_ENTROPY), the score K - c (static) or
 * K - c * n_hi (dynamic), and the decision of the chosen policy:
 *   S2D2_ROUTE_MIN_SPAN     |C_t| >= tau_span
 *   S2D2_ROUTE_SCORE        score >= tau_score
 *   S2D2_ROUTE_HYSTERESIS   state ON and score < tau_off -> OFF; state OFF and score >= tau_on -> ON; verify iff ON
 * A sequence whose block has no [MASK] is never verified.  fp32 arithmetic, products and sum taken left to right.
 * Outputs (device, caller-owned, [N]):
 *   do_verify        1 = run the verifier for this sequence, 0 = fall back to the threshold commit of Alg. 2;
 *                    pass it as s2d2_params.active to s2d2_verify / s2d2_accept
 *   khat, score      K and the score (score is computed under every policy)
 *   unmask_fallback  the draft's threshold set where do_verify == 0, else 0: a copy of the draft outputs with
 *                    `unmask` pointing here makes s2d2_commit_threshold act on exactly the sequences that fell back
 * hysteresis: device [N], in/out, 1 = ON, 0 = OFF; read and written only under S2D2_ROUTE_HYSTERESIS (may be NULL
 * otherwise).  Errors: S2D2_EINVAL for a NULL argument, an unknown policy or estimator, tau_span < 0. */
#define S2D2_ROUTE_MIN_SPAN 0
#define S2D2_ROUTE_SCORE 1
#define S2D2_ROUTE_HYSTERESIS 2
#define S2D2_EST_MARGIN 0
#define S2D2_EST_ENTROPY 1
typedef struct {
  int32_t policy, estimator;
  int32_t dynamic;      /* 0: score = K - c; 1: score = K - c * n_hi */
  int32_t tau_span;
  float tau_score, tau_on, tau_off;
  float c, beta, tau_margin;
} s2d2_route_params;
typedef struct {
  int32_t* do_verify;
  float* khat;
  float* score;
  uint64_t* unmask_fallback;
} s2d2_route_out;
int32_t s2d2_route(s2d2_ctx* ctx, int32_t N, int32_t B, const s2d2_route_params* rp, const s2d2_draft_out* draft,
                   int32_t* hysteresis, const s2d2_route_out* out);

/* Synchronises the context's stream and reports a sticky device-side failure: S2D2_ELAUNCH if a workgroup of the
 * down projection waited in vain for the partial sums of the workgroup it shares K with (the results of that
 * forward are then invalid); S2D2_OK otherwise.  No kernel of the library waits unboundedly. */
int32_t s2d2_status(s2d2_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* S2D2_H */
