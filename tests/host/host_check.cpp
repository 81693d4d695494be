// Host-side argument validation and size arithmetic of libs2d2 under AddressSanitizer / UndefinedBehaviorSanitizer.
// Links the library's objects with api.hip rebuilt with -fsanitize=address,undefined on the host side (device code
// is not instrumented and never launched here: no call below gets past its argument checks).  Exits 0 if every
// call returned what its contract says; the sanitizers abort the process on a finding.
#include <climits>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/s2d2.h"
#include "../../include/s2d2_aux.h"

static int g_bad = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond, s2d2_last_error()); ++g_bad; } } while (0)

static s2d2_model_desc dense(int layers, int d, int hq, int hkv, int D, int ffn, int vocab, int dtype) {
  s2d2_model_desc m;
  std::memset(&m, 0, sizeof m);
  m.n_layers = layers; m.d_model = d; m.n_q_heads = hq; m.n_kv_heads = hkv; m.head_dim = D; m.d_ffn = ffn; m.vocab = vocab;
  m.dtype = dtype; m.mask_id = vocab - 1; m.rope_theta = 1e6f; m.rms_eps = 1e-6f;
  return m;
}

int main() {
  // ---- the shapes of the benchmark configurations: sizes are positive and grow with batch and block ----
  const s2d2_model_desc shapes[] = {
      dense(2, 256, 4, 2, 64, 512, 1000, S2D2_F32),
      dense(28, 2048, 16, 8, 128, 6144, 151936, S2D2_BF16),
      dense(36, 2560, 32, 8, 128, 9728, 151936, S2D2_BF16),
      dense(36, 4096, 32, 8, 128, 12288, 151936, S2D2_BF16),
  };
  for (const s2d2_model_desc& m : shapes) {
    const int64_t w1 = s2d2_workspace_bytes(&m, 1, 4), w2 = s2d2_workspace_bytes(&m, 16, 16), w3 = s2d2_workspace_bytes(&m, 1024, 64);
    EXPECT(w1 > 0 && w2 > w1 && w3 > w2);
    EXPECT(s2d2_packed_bytes(&m) >= 0);
    EXPECT(s2d2_stage_rows(16, 16) == 3 * 16 * 16);
  }
  s2d2_model_desc moe = dense(20, 2048, 16, 4, 128, 0, 157184, S2D2_BF16);
  moe.n_experts = 64; moe.top_k = 8; moe.d_expert = 1024;
  EXPECT(s2d2_workspace_bytes(&moe, 32, 32) > 0 && s2d2_packed_bytes(&moe) > 0);

  // ---- every integer field at its extremes: an error code or a size, never a crash or an overflow ----
  const int32_t extremes[] = {INT32_MIN, -1, 0, 1, 31, 32, 33, 65535, 65536, 1 << 24, INT32_MAX - 1, INT32_MAX};
  const size_t n_fields = 14;
  for (size_t f = 0; f < n_fields; ++f)
    for (int32_t v : extremes)
      for (int base = 0; base < 2; ++base) {
        s2d2_model_desc m = base ? moe : shapes[3];
        int32_t* fields = &m.n_layers;   // the 14 leading int32 fields of the struct, in declaration order
        fields[f] = v;
        const int64_t w = s2d2_workspace_bytes(&m, 1024, S2D2_MAX_BLOCK), p = s2d2_packed_bytes(&m);
        EXPECT(w != 0 && p >= -4);
        EXPECT((w < 0) == (p < 0) || w > 0);   // a description the packing accepts is accepted by the sizing as well
      }
  for (int32_t nb : extremes)
    for (int32_t bl : extremes) {
      const int64_t w = s2d2_workspace_bytes(&shapes[1], nb, bl);
      const bool ok = nb >= 1 && nb <= 1024 && bl >= 1 && bl <= S2D2_MAX_BLOCK;
      EXPECT(ok ? w > 0 : w == S2D2_EINVAL);
      const int64_t r = s2d2_stage_rows(nb, bl);
      EXPECT(ok ? r == 3LL * nb * bl : r < 0);
    }
  s2d2_model_desc nanm = shapes[1];
  nanm.rope_theta = 0.0f / 0.0f * 0.0f;
  EXPECT(s2d2_workspace_bytes(&nanm, 1, 4) == S2D2_EINVAL);
  EXPECT(s2d2_workspace_bytes(nullptr, 1, 4) == S2D2_EINVAL && s2d2_packed_bytes(nullptr) == S2D2_EINVAL);

  // ---- s2d2_create refuses bad arguments before it looks for a device ----
  s2d2_ctx* ctx = (s2d2_ctx*)(uintptr_t)1;
  std::vector<s2d2_layer_weights> layers(shapes[1].n_layers);
  std::memset(layers.data(), 0, layers.size() * sizeof(s2d2_layer_weights));
  s2d2_weights w;
  std::memset(&w, 0, sizeof w);
  EXPECT(s2d2_create(&shapes[1], &w, 1, 4, nullptr, nullptr, 0, nullptr, 0, nullptr) == S2D2_EINVAL);
  EXPECT(s2d2_create(&shapes[1], &w, 1, 4, nullptr, nullptr, 0, nullptr, 0, &ctx) == S2D2_EINVAL && ctx == nullptr);
  EXPECT(s2d2_create(nullptr, &w, 1, 4, nullptr, nullptr, 0, nullptr, 0, &ctx) == S2D2_EINVAL);
  EXPECT(s2d2_create(&shapes[1], nullptr, 1, 4, nullptr, nullptr, 0, nullptr, 0, &ctx) == S2D2_EINVAL);
  EXPECT(s2d2_create(&shapes[1], &w, 0, 4, nullptr, nullptr, 0, nullptr, 0, &ctx) == S2D2_EINVAL);
  EXPECT(s2d2_create(&shapes[1], &w, 1, S2D2_MAX_BLOCK + 1, nullptr, nullptr, 0, nullptr, 0, &ctx) == S2D2_EINVAL);
  // plausible (fake, never dereferenced) device pointers, all aligned: the layer array is read, a missing matrix is found
  void* fake = (void*)(uintptr_t)0x7f0000000000ull;
  w.embed = fake; w.unembed = fake; w.norm_f = (const float*)fake; w.layers = layers.data();
  EXPECT(s2d2_create(&shapes[1], &w, 1, 4, nullptr, fake, 1 << 20, nullptr, 0, &ctx) == S2D2_EINVAL);
  for (s2d2_layer_weights& L : layers) { L.norm1 = L.norm2 = (const float*)fake; L.wqkv = L.wo = L.wgu = L.wdown = fake; }
  layers[5].wo = (void*)(uintptr_t)0x7f0000000008ull;   // not 16-byte aligned
  EXPECT(s2d2_create(&shapes[1], &w, 1, 4, nullptr, fake, 1 << 20, nullptr, 0, &ctx) == S2D2_EINVAL);
  layers[5].wo = fake;
  EXPECT(s2d2_create(&shapes[1], &w, 1, 4, nullptr, (void*)(uintptr_t)0x7f0000000010ull, 1 << 20, nullptr, 0, &ctx) == S2D2_EINVAL);   // workspace not 256-byte aligned
  EXPECT(s2d2_create(&shapes[1], &w, 1, 4, nullptr, fake, 1 << 20, nullptr, 0, &ctx) == S2D2_ENOSPC);   // workspace too small
  EXPECT(s2d2_create(&moe, &w, 1, 4, nullptr, fake, (size_t)1 << 40, nullptr, 0, &ctx) == S2D2_EINVAL);   // MoE weights missing

  // ---- calls on a NULL context or with NULL structures ----
  s2d2_kv_view kv; s2d2_block_state st; s2d2_params prm; s2d2_draft_out d; s2d2_verify_out v; s2d2_accept_out a; s2d2_route_params rp; s2d2_profile pf;
  std::memset(&kv, 0, sizeof kv); std::memset(&st, 0, sizeof st); std::memset(&prm, 0, sizeof prm); std::memset(&d, 0, sizeof d);
  std::memset(&v, 0, sizeof v); std::memset(&a, 0, sizeof a); std::memset(&rp, 0, sizeof rp); std::memset(&pf, 0, sizeof pf);
  EXPECT(s2d2_draft(nullptr, &kv, &st, 1, 4, &prm, &d) == S2D2_EINVAL);
  EXPECT(s2d2_verify(nullptr, &kv, &st, 1, 4, &prm, &d, &v) == S2D2_EINVAL);
  EXPECT(s2d2_accept(nullptr, &st, 1, 4, &prm, &d, &v, &a) == S2D2_EINVAL);
  EXPECT(s2d2_kv_append(nullptr, &kv, 1, 4, &d, &v, nullptr) == S2D2_EINVAL);
  EXPECT(s2d2_block_complete(nullptr, &kv, &st, 1, 4, &v, 0) == S2D2_EINVAL);
  EXPECT(s2d2_block_advance(nullptr, &kv, &st, 1, 4, nullptr) == S2D2_EINVAL);
  EXPECT(s2d2_commit_threshold(nullptr, &st, 1, 4, &d) == S2D2_EINVAL);
  EXPECT(s2d2_route(nullptr, 1, 4, &rp, &d, nullptr, nullptr) == S2D2_EINVAL);
  EXPECT(s2d2_set_stream(nullptr, nullptr) == S2D2_EINVAL);
  EXPECT(s2d2_status(nullptr) == S2D2_EINVAL);
  EXPECT(s2d2_destroy(nullptr) == S2D2_EINVAL || s2d2_destroy(nullptr) == S2D2_OK);
  EXPECT(s2d2_profile_start(nullptr, 16) == S2D2_EINVAL && s2d2_profile_stop(nullptr, &pf) == S2D2_EINVAL);
  // the entry point without a context checks its limits before it touches the device
  EXPECT(s2d2_accept_static(nullptr, 1 << 19, &st, 1, 4, &prm, &d, &v, &a) == S2D2_ENOSPC);
  EXPECT(s2d2_accept_static(nullptr, 1000, &st, 129, 4, &prm, &d, &v, &a) == S2D2_ENOSPC);
  EXPECT(s2d2_accept_static(nullptr, 1000, nullptr, 1, 4, &prm, &d, &v, &a) == S2D2_EINVAL);
  EXPECT(std::strlen(s2d2_version()) > 0 && s2d2_last_error() != nullptr);

  std::printf("host_check: %d failed expectation(s)\n", g_bad);
  return g_bad ? 1 : 0;
}
