/*
 * s2d2_aux.h - inspection and measurement aids of libs2d2.  NOT part of the decoding step's boundary (that is
 * s2d2.h): nothing here is needed to run the method.  The parity tests and the benchmark use these calls to hold
 * the CPU reference to the device's expert choices, to run the vocabulary stage alone on given logits, to look at
 * intermediate activations, and to time kernel launches by class.  Layouts and semantics may change.
 */
#ifndef S2D2_AUX_H
#define S2D2_AUX_H

#include "s2d2.h"

#ifdef __cplusplus
extern "C" {
#endif

/* MoE models: the experts chosen by the router in the most recent forward (draft or verifier),
 * out = device [n_layers, rows, top_k] int32 for the first `rows` window rows (window rows are packed
 * sequence after sequence: leading causal rows, drafted rows, then [MASK] copies).  The parity
 * tests use it to hold the oracle to the same routing where a router score is tied to rounding. */
int32_t s2d2_moe_choices(s2d2_ctx* ctx, int32_t rows, int32_t* out /* device */);

/* Debugging aid: device address of an internal activation buffer of the most recent forward
 * ("h" fp32 residual rows [rows, d]; "a" operand of the next norm; "q", "o", "ffn", "kwin", "vwin", "ss").
 * Contents are those of the last layer that ran; layouts are internal and may change. */
int32_t s2d2_debug_buffer(s2d2_ctx* ctx, const char* name, void** ptr);

/* Vocabulary stage alone on caller-provided logits (same kernels the calls above use):
 * draft statistics for `rows` fp32 logit rows of width V.  Outputs are [rows]. */
int32_t s2d2_vocab_draft_stats(s2d2_ctx* ctx, const float* logits, int32_t rows, int32_t* xhat,
                               float* p, float* lse, float* margin, float* entropy_n);
/* Verifier side: q[r] = softmax(logits_ver[r])[token[r]] and lse[r]. */
int32_t s2d2_vocab_score(s2d2_ctx* ctx, const float* logits_ver, int32_t rows,
                         const int32_t* token, float* q, float* lse);

/* Measurement aid (not part of the method): while profiling is on, the kernel launches of a step are
 * timed with HIP events on the context's stream and attributed to a class.
 * s2d2_profile_stop synchronises the stream, sums the event times and turns profiling off.
 *   launches    kernel launches of the class
 *   ms          summed kernel durations: the two events of a launch are stamped by the dispatch itself
 *               (hipExtLaunchKernelGGL), i.e. they read what a kernel trace reads for that launch
 *   bytes       algorithmic HBM bytes of those launches: weight matrix once for a GEMM, K and V
 *               of the cached prefix once for attention, the fp32 logit rows once for the
 *               vocabulary kernels (window rows and tiny outputs are not counted)
 * Classes: 0 all GEMMs, 1 attention, 2 vocabulary, 3 everything else; 4-8 split class 0 by kind: 4 QKV projection,
 * 5 output projection, 6 gate / up (dense or grouped experts), 7 down projection (dense or grouped experts),
 * 8 unembedding (the MoE router GEMM is counted in class 0 only). */
#define S2D2_PROFILE_CLASSES 9
typedef struct {
  int64_t launches;
  double ms;
  double bytes;
  double flops;     /* GEMM class: 2 x rows x N x K per launch on the rows a fresh block gives (N*B draft rows, 2*N*B
                       verifier rows, N*B logit rows), the method's flops counted once (a second activation plane
                       doubles the instructions issued, not this figure); 0 for the other classes */
  double max_ms;    /* longest single launch of the class */
} s2d2_profile;
int32_t s2d2_profile_start(s2d2_ctx* ctx, int32_t max_launches);
int32_t s2d2_profile_stop(s2d2_ctx* ctx, s2d2_profile* out /* host [S2D2_PROFILE_CLASSES] */);

#ifdef __cplusplus
}
#endif
#endif /* S2D2_AUX_H */
