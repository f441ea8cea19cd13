// Host-side exercise of the C ABI for a sanitizer build (AddressSanitizer + UndefinedBehaviorSanitizer on the host
// code only): every entry point is driven through its argument validation, the workspace map and the context
// life cycle with device pointers that are never dereferenced on the host.  No GPU is needed: nothing is launched.
// Exit status 0 = every call returned what it should; the sanitizers abort the process on a finding.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <vector>
#include "../../include/dllm.h"

static int failures = 0;
#define EXPECT(call, want)                                                            \
  do {                                                                                \
    const long got_ = (long)(call);                                                   \
    if (got_ != (long)(want)) { printf("line %d: got %ld, want %ld\n", __LINE__, got_, (long)(want)); ++failures; } \
  } while (0)

static dllm_config tiny_cfg() {
  dllm_config c;
  memset(&c, 0, sizeof(c));
  c.n_layers = 2; c.d_model = 256; c.n_q_heads = 4; c.n_kv_heads = 4; c.head_dim = 64; c.d_ff = 688;
  c.vocab = 4096; c.mask_id = 4095; c.rms_eps = 1e-5f; c.rope_base = 10000.f; c.dtype = DLLM_F32;
  c.page_tokens = 16; c.max_pages_per_seq = 8; c.n_pages = 8; c.max_batch = 2; c.max_q = 32; c.max_tokens = 128;
  return c;
}

int main() {
  void* const p = (void*)0x3000;          // stands for device memory; the host never reads it
  int32_t* const ip = (int32_t*)p;
  float* const fp = (float*)p;
  for (int dtype = 0; dtype < 2; ++dtype) {
    dllm_config cfg = tiny_cfg();
    cfg.dtype = dtype;
    if (dtype == DLLM_BF16) { cfg.d_ff = 688; cfg.n_kv_heads = 2; }
    const size_t ws = dllm_workspace_bytes(&cfg), kv = dllm_kv_pool_bytes(&cfg);
    EXPECT(ws > 0 && kv > 0, 1);
    std::vector<dllm_layer_w> lw(cfg.n_layers);
    for (auto& l : lw) l = dllm_layer_w{p, p, p, p, p, p, p, p, p};
    dllm_weights w{p, p, p, lw.data()};
    dllm_ctx* ctx = nullptr;
    void* const wsp = (void*)(0x20000 * 256);
    EXPECT(dllm_create(&ctx, &cfg, &w, p, kv - 1, wsp, ws), DLLM_ENOSPACE);
    EXPECT(dllm_create(&ctx, &cfg, &w, p, kv, wsp, ws - 1), DLLM_ENOSPACE);
    EXPECT(dllm_create(&ctx, &cfg, &w, nullptr, kv, wsp, ws), DLLM_EINVAL);
    EXPECT(dllm_create(&ctx, &cfg, &w, p, kv, (char*)wsp + 8, ws), DLLM_EINVAL);
    EXPECT(dllm_create(nullptr, &cfg, &w, p, kv, wsp, ws), DLLM_EINVAL);
    { dllm_config bad = cfg; bad.head_dim = 48; EXPECT(dllm_workspace_bytes(&bad), 0); EXPECT(dllm_create(&ctx, &bad, &w, p, kv, wsp, ws), DLLM_ESHAPE); }
    { dllm_config bad = cfg; bad.mask_id = cfg.vocab; EXPECT(dllm_kv_pool_bytes(&bad), 0); }
    { dllm_config bad = cfg; bad.max_batch = 1 << 20; bad.max_q = 1 << 20; EXPECT(dllm_workspace_bytes(&bad), 0); }
    lw[1].wo = nullptr;
    EXPECT(dllm_create(&ctx, &cfg, &w, p, kv, wsp, ws), DLLM_EINVAL);
    lw[1].wo = p;
    EXPECT(dllm_create(&ctx, &cfg, &w, p, kv, wsp, ws), DLLM_OK);
    if (!ctx) { printf("no context\n"); return 2; }
    // steps
    EXPECT(dllm_denoise_step(ctx, nullptr, 0, 32, 64, ip, ip, ip, ip, fp, nullptr), DLLM_EINVAL);
    EXPECT(dllm_denoise_step(ctx, nullptr, 3, 32, 64, ip, ip, ip, ip, fp, nullptr), DLLM_ESHAPE);
    EXPECT(dllm_denoise_step(ctx, nullptr, 1, 33, 64, ip, ip, ip, ip, fp, nullptr), DLLM_ESHAPE);
    EXPECT(dllm_denoise_step(ctx, nullptr, 1, 32, 97, ip, ip, ip, ip, fp, nullptr), DLLM_ESHAPE);
    EXPECT(dllm_denoise_step(ctx, nullptr, 1, 32, -1, ip, ip, ip, ip, fp, nullptr), DLLM_EINVAL);
    EXPECT(dllm_denoise_step(ctx, nullptr, 1, 32, 64, nullptr, ip, ip, ip, fp, nullptr), DLLM_EINVAL);
    EXPECT(dllm_denoise_step(nullptr, nullptr, 1, 32, 64, ip, ip, ip, ip, fp, nullptr), DLLM_EINVAL);
    EXPECT(dllm_denoise_step_var(ctx, nullptr, 1, 32, 64, ip, ip, nullptr, ip, ip, fp, nullptr), DLLM_EINVAL);
    EXPECT(dllm_denoise_step_live(ctx, nullptr, 1, 32, 64, ip, ip, nullptr, nullptr, ip, ip, fp, nullptr), DLLM_EINVAL);
    EXPECT(dllm_denoise_step_static(ctx, nullptr, 1, 33, 64, ip, ip, ip, ip, fp, nullptr), DLLM_ESHAPE);
    EXPECT(dllm_debug_logits(ctx, nullptr, 1, 32, 64, ip, ip, ip, nullptr), DLLM_EINVAL);
    EXPECT(dllm_debug_hidden(ctx, nullptr, 1, 32, 64, ip, ip, ip, 3, fp), DLLM_EINVAL);
    // packed forwards
    EXPECT(dllm_prefill_kv(ctx, nullptr, 1, 129, 129, ip, ip, nullptr, ip), DLLM_ESHAPE);
    EXPECT(dllm_prefill_kv(ctx, nullptr, 1, 0, 0, ip, ip, nullptr, ip), DLLM_EINVAL);
    EXPECT(dllm_prefill_kv(ctx, nullptr, 1, 64, 65, ip, ip, nullptr, ip), DLLM_EINVAL);
    EXPECT(dllm_prefill_kv(ctx, nullptr, 3, 64, 64, ip, ip, nullptr, ip), DLLM_ESHAPE);
    EXPECT(dllm_refresh_cache(ctx, nullptr, 1, 64, 64, ip, ip, nullptr, ip, ip, fp, nullptr), DLLM_EINVAL);
    // selection, state machine, bookkeeping
    EXPECT(dllm_unmask(ctx, nullptr, 1, 32, 32, ip, ip, fp, 0.9f, -1, nullptr, nullptr), DLLM_EINVAL);
    EXPECT(dllm_unmask(ctx, nullptr, 1, 32, 5, ip, ip, fp, 0.9f, 1, nullptr, nullptr), DLLM_EINVAL);
    EXPECT(dllm_unmask(ctx, nullptr, 1, 4096, 2048, ip, ip, fp, 0.9f, 1, nullptr, nullptr), DLLM_ESHAPE);
    EXPECT(dllm_unmask_entropy(ctx, nullptr, 1, 32, 32, ip, ip, nullptr, 0.45f, 1, nullptr, nullptr), DLLM_EINVAL);
    EXPECT(dllm_unmask_blocks(ctx, nullptr, 1, 64, 32, ip, ip, fp, 0.45f, 1, nullptr, nullptr, nullptr), DLLM_EINVAL);
    EXPECT(dllm_unmask_traced(ctx, nullptr, 1, 32, 32, ip, ip, fp, 2.0f, 0, 1, 1, nullptr, nullptr, nullptr), DLLM_EINVAL);
    EXPECT(dllm_fsm_update(ctx, nullptr, 1, 257, 32, ip, ip, ip, 0.1, 0.95, 1, 0, nullptr, nullptr), DLLM_ESHAPE);
    EXPECT(dllm_fsm_update(ctx, nullptr, 1, 8, 32, ip, ip, ip, 0.1, 0.95, -1, 0, nullptr, nullptr), DLLM_EINVAL);
    EXPECT(dllm_fsm_plan(ctx, nullptr, 1, 8, 32, ip, ip, nullptr, -1, ip, ip, ip), DLLM_EINVAL);
    EXPECT(dllm_fsm_plan(ctx, nullptr, 1, 8, 32, ip, ip, nullptr, 4, nullptr, ip, ip), DLLM_EINVAL);
    EXPECT(dllm_fsm_window(ctx, nullptr, 1, 8, 32, 0, ip, ip, ip, 0, ip, ip, ip, ip, ip), DLLM_EINVAL);
    EXPECT(dllm_fsm_scatter(ctx, nullptr, 1, 8, 32, 2, ip, ip, nullptr, ip), DLLM_EINVAL);
    EXPECT(dllm_fsm_round_windows(ctx, nullptr, 1, 8, 32, 2, ip, ip, ip, nullptr, 0, ip, ip, ip, ip, ip, ip), DLLM_EINVAL);
    EXPECT(dllm_fsm_round_windows(ctx, nullptr, 1, 8, 32, 2, ip, ip, ip, ip, cfg.mask_id, ip, ip, ip, ip, ip, ip), DLLM_EINVAL);
    EXPECT(dllm_fsm_pack(ctx, nullptr, 1, 8, 32, 2, 0, 128, 128, ip, ip, ip, ip, ip, ip, 0, ip, ip, ip), DLLM_EINVAL);
    EXPECT(dllm_fsm_pack(ctx, nullptr, 1, 300, 32, 2, 64, 128, 128, ip, ip, ip, ip, ip, ip, 0, ip, ip, ip), DLLM_ESHAPE);
    EXPECT(dllm_fsm_unpack(ctx, nullptr, 1, 0, 128, ip, ip, ip, ip, ip, fp, nullptr, ip, fp, nullptr), DLLM_EINVAL);
    EXPECT(dllm_refresh_cache_dev(ctx, nullptr, 1, 64, 64, ip, ip, nullptr, ip, ip, fp, nullptr), DLLM_EINVAL);
    EXPECT(dllm_refresh_cache_dev(ctx, nullptr, 1, 129, 129, ip, ip, ip, ip, ip, fp, nullptr), DLLM_ESHAPE);
    EXPECT(dllm_noisy_sequence(ctx, nullptr, 1, 32, ip, ip, ip, 8, 1.5, ip), DLLM_EINVAL);
    EXPECT(dllm_eos_scan(ctx, nullptr, 1, 32, ip, 5, ip, nullptr, ip, nullptr), DLLM_EINVAL);
    EXPECT(dllm_gather_rows(ctx, nullptr, 2, 4, ip, ip, ip, ip, 0), DLLM_EINVAL);
    EXPECT(dllm_scatter_rows(ctx, nullptr, 0, 4, ip, ip, ip, ip + 64), DLLM_EINVAL);
    EXPECT(dllm_set_kernel_mode(ctx, 7), DLLM_EINVAL);
    EXPECT(dllm_set_kernel_mode(ctx, 1), DLLM_OK);
    EXPECT(dllm_read_status(ctx, nullptr, nullptr), DLLM_EINVAL);
    EXPECT(dllm_profile_read(ctx, nullptr, 0, nullptr, nullptr, nullptr), DLLM_EINVAL);
    if (dtype == DLLM_BF16) {
      EXPECT(dllm_packed_weight_bytes(&cfg) > 0, 1);
      EXPECT(dllm_pack_weights(ctx, nullptr, nullptr, 0), DLLM_EINVAL);
      EXPECT(dllm_pack_weights(ctx, nullptr, (char*)wsp + 16, dllm_packed_weight_bytes(&cfg)), DLLM_EINVAL);
      EXPECT(dllm_pack_weights(ctx, nullptr, wsp, dllm_packed_weight_bytes(&cfg) - 1), DLLM_ENOSPACE);
    } else {
      EXPECT(dllm_packed_weight_bytes(&cfg), 0);
      EXPECT(dllm_pack_weights(ctx, nullptr, wsp, 1 << 20), DLLM_ESHAPE);
    }
    EXPECT(strlen(dllm_strerror(DLLM_ESHAPE)) > 0, 1);
    EXPECT(strlen(dllm_last_hip_error(ctx)), 0);
    dllm_destroy(ctx);
  }
  dllm_destroy(nullptr);
  // a context too large for the library's own scratch array
  {
    dllm_config cfg = tiny_cfg();
    cfg.max_tokens = 16384;
    std::vector<dllm_layer_w> lw(cfg.n_layers, dllm_layer_w{p, p, p, p, p, p, p, p, p});
    dllm_weights w{p, p, p, lw.data()};
    dllm_ctx* ctx = nullptr;
    EXPECT(dllm_create(&ctx, &cfg, &w, p, dllm_kv_pool_bytes(&cfg), (void*)(0x20000 * 256), dllm_workspace_bytes(&cfg)), DLLM_OK);
    EXPECT(dllm_workspace_bytes(&cfg) > dllm_static_scratch_bytes(), 1);
    EXPECT(dllm_denoise_step_static(ctx, nullptr, 1, 32, 64, ip, ip, ip, ip, fp, nullptr), DLLM_ENOSPACE);
    dllm_destroy(ctx);
  }
  printf("host check: %d failure(s)\n", failures);
  return failures ? 1 : 0;
}
