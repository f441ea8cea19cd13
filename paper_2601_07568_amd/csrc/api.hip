// extern "C" surface of the library: argument validation (host only, before anything is
// launched), workspace map, and the chain of launches that makes up each call.
#include "common.h"
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

using namespace dllm;

namespace dllm {
hipError_t launch_set_i32(hipStream_t s, int32_t* p, int n, int32_t v);
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static bool config_ok(const dllm_config* c) {
  if (!c) return false;
  if (c->n_layers < 0 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ff < 1) return false;
  if (c->vocab < 2 || c->mask_id < 0 || c->mask_id >= c->vocab) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->n_q_heads % c->n_kv_heads != 0) return false;
  if (c->dtype != DLLM_F32 && c->dtype != DLLM_BF16) return false;
  if (c->dtype == DLLM_BF16 && (c->d_model % 8 != 0 || c->d_ff % 8 != 0)) return false;
  if (c->page_tokens < 1 || c->max_pages_per_seq < 1 || c->n_pages < 1) return false;
  if (c->max_batch < 1 || c->max_q < 1 || c->max_tokens < 0) return false;
  if (!(c->rms_eps >= 0.f) || !(c->rope_base > 1.f)) return false;
  if ((int64_t)c->max_batch * c->max_q > (1 << 20) || c->max_tokens > (1 << 22)) return false;
  return true;
}

static bool build_map(const dllm_config* c, Workspace* m) {
  if (!config_ok(c)) return false;
  const size_t es = elem_size(*c);
  const size_t t_step = (size_t)c->max_batch * c->max_q;
  const size_t t_max = t_step > (size_t)c->max_tokens ? t_step : (size_t)c->max_tokens;
  const size_t dq = (size_t)c->n_q_heads * c->head_dim, dkv = (size_t)c->n_kv_heads * c->head_dim;
  const size_t half = c->head_dim / 2;
  m->t_max = (int64_t)t_max;
  m->t_step = (int64_t)t_step;
  m->r_max = (int64_t)t_step;
  m->n_vtiles = (c->vocab + LM_TILE_N - 1) / LM_TILE_N;
  m->max_splits = ATTN_MAX_SPLITS;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  m->status = take(64);
  m->x = take(t_max * c->d_model * 4);
  m->xn = take((t_max + 16) * ((size_t)c->d_model + 128) * es);
  m->q32 = take(t_max * dq * 4);
  m->k32 = take(t_max * dkv * 4);
  m->q = take(t_max * dq * es);
  m->tpad = c->max_tokens > 0 ? (int64_t)c->max_tokens + 32 * (int64_t)c->max_batch : 0;
  m->v = take(t_max * dkv * es);
  // 64 rows / 64 keys of slack: the staged attention reads whole 64-key blocks, also a sequence's last one
  m->kpack = take(((size_t)m->tpad + 64) * dkv * es);
  m->vpack = take(((size_t)m->tpad * dkv + 64) * es);
  m->cu_pad = take(((size_t)c->max_batch + 1) * 4);
  m->o = take((t_max + 16) * (dq + 128) * es);
  m->g_bytes = t_max * c->d_ff * 4;
  m->g = take(m->g_bytes);
  m->u = take(t_max * c->d_ff * 4);
  m->h = take((t_max + 16) * ((size_t)c->d_ff + 128) * es);
  m->rope_cos = take(t_max * half * 4);
  m->rope_sin = take(t_max * half * 4);
  m->tok_seq = take(t_max * 4);
  m->tok_pos = take(t_max * 4);
  m->rows = take((size_t)m->r_max * 4);
  m->lm_part = take((size_t)m->r_max * ((c->vocab + 63) / 64) * 4 * 4);   // finest split: 64 columns per partial
  m->attn_rows = (int64_t)t_step * c->n_q_heads * 8;
  if (m->attn_rows < 65536) m->attn_rows = 65536;
  m->attn_part = take(c->dtype == DLLM_BF16 ? (size_t)m->attn_rows * (c->head_dim + 2) * 4 : 0);
  if (c->dtype != DLLM_BF16) m->attn_rows = 0;
  m->len_safe = take(((size_t)c->max_batch + 1) * 4);
  m->q_valid_eff = take((size_t)c->max_batch * 4);
  m->rscale = take(t_max * 4);
  m->ss = take((size_t)64 * ((((size_t)c->d_model + 15) / 16 + 3) / 4 * 4) * 4);
  m->delta_stride = (int64_t)SK_MAX_ROWS * c->d_model;
  m->lg_delta_rows = c->dtype == DLLM_BF16 ? (int64_t)(t_max < (size_t)LG_DELTA_ROWS ? t_max : (size_t)LG_DELTA_ROWS) : 0;
  m->lg_delta_stride = m->lg_delta_rows * c->d_model;
  {
    size_t lg_floats = (size_t)LG_MAX_DELTA * m->lg_delta_stride;
    m->delta = take(c->dtype == DLLM_BF16 ? lg_floats * 4 : 0);
  }
  m->qkvp_stride = m->lg_delta_rows * (int64_t)(dq + 2 * dkv);
  m->qkvp_rows = (int64_t)LG_QKV_SPLITS * m->lg_delta_rows > (int64_t)t_max ? (int64_t)LG_QKV_SPLITS * m->lg_delta_rows : (int64_t)t_max;
  if (c->dtype != DLLM_BF16) m->qkvp_rows = 0;
  m->qkvp = take((size_t)m->qkvp_rows * (dq + 2 * dkv) * 4);
  m->scratch_bytes = 0;
  m->scratch = take(m->scratch_bytes);
  m->total = off;
  return true;
}

extern "C" size_t dllm_workspace_bytes(const dllm_config* cfg) {
  Workspace m;
  return build_map(cfg, &m) ? m.total : 0;
}

extern "C" size_t dllm_kv_pool_bytes(const dllm_config* cfg) {
  if (!config_ok(cfg)) return 0;
  return (size_t)cfg->n_layers * 2 * kv_slab_elems(*cfg) * elem_size(*cfg);
}

static int hip_fail(dllm_ctx* c, hipError_t e, const char* where) {
  snprintf(c->hip_error, sizeof(c->hip_error), "%s: %s", where, hipGetErrorString(e));
  return DLLM_EHIP;
}
#define TRY(call, where)                        \
  do {                                          \
    hipError_t e_ = (call);                     \
    if (e_ != hipSuccess) return hip_fail(c, e_, where); \
  } while (0)

extern "C" int dllm_create(dllm_ctx** out, const dllm_config* cfg, const dllm_weights* w, void* kv_pool,
                           size_t kv_pool_bytes, void* workspace, size_t workspace_bytes) {
  if (!out) return DLLM_EINVAL;
  *out = nullptr;
  if (!cfg || !w || !kv_pool || !workspace) return DLLM_EINVAL;
  Workspace m;
  if (!build_map(cfg, &m)) return DLLM_ESHAPE;
  if (!w->tok_emb || !w->final_norm || !w->lm_head) return DLLM_EINVAL;
  if (cfg->n_layers > 0 && !w->layers) return DLLM_EINVAL;
  for (int l = 0; l < cfg->n_layers; ++l) {
    const dllm_layer_w& L = w->layers[l];
    if (!L.attn_norm || !L.wq || !L.wk || !L.wv || !L.wo || !L.mlp_norm || !L.w_gate || !L.w_up || !L.w_down)
      return DLLM_EINVAL;
  }
  if (((uintptr_t)workspace & 255) != 0) return DLLM_EINVAL;
  if (workspace_bytes < m.total || kv_pool_bytes < dllm_kv_pool_bytes(cfg)) return DLLM_ENOSPACE;
  dllm_ctx* c = (dllm_ctx*)calloc(1, sizeof(dllm_ctx));
  if (!c) return DLLM_ENOSPACE;
  c->cfg = *cfg;
  c->layers = (dllm_layer_w*)calloc(cfg->n_layers > 0 ? cfg->n_layers : 1, sizeof(dllm_layer_w));
  if (!c->layers) { free(c); return DLLM_ENOSPACE; }
  for (int l = 0; l < cfg->n_layers; ++l) c->layers[l] = w->layers[l];
  c->tok_emb = w->tok_emb;
  c->final_norm = w->final_norm;
  c->lm_head = w->lm_head;
  c->kv_pool = (char*)kv_pool;
  c->ws = (char*)workspace;
  c->map = m;
  c->kernel_mode = 0;
  if (cfg->dtype == DLLM_BF16) {
    // raising two kernels' LDS limits; a failure (e.g. no device in this process) is not an error of the call: the
    // launchers check the flags these leave and take the kernels that need no raised limit
    const hipError_t e1 = init_gemm_t256();      // without it the 128-row kernels serve every size
    const hipError_t e2 = init_attn_kernels();   // without it every wave of the batch-1 attention writes its own partial
    // such a failure must not surface later as the "last error" of an unrelated launch
    if (e1 != hipSuccess || e2 != hipSuccess) (void)hipGetLastError();
  }
  *out = c;
  return DLLM_OK;
}

static void prof_free(dllm_ctx* c) {
  if (c->prof_ev) {
    for (int i = 0; i < 2 * c->prof_cap; ++i) (void)hipEventDestroy(c->prof_ev[i]);
    free(c->prof_ev);
    free(c->prof_cls);
    free(c->prof_bytes);
  }
  c->prof_ev = nullptr; c->prof_cls = nullptr; c->prof_bytes = nullptr;
  c->prof_on = c->prof_n = c->prof_cap = 0;
}

static size_t align256(size_t v) { return (v + 255) / 256 * 256; }

extern "C" size_t dllm_packed_weight_bytes(const dllm_config* f) {
  if (!config_ok(f) || f->dtype != DLLM_BF16) return 0;
  const int dq = f->n_q_heads * f->head_dim, dkv = f->n_kv_heads * f->head_dim;
  size_t per_layer = align256(packed_weight_bytes(dq, f->d_model)) + 2 * align256(packed_weight_bytes(dkv, f->d_model)) +
                     align256(packed_weight_bytes(f->d_model, dq)) + 2 * align256(packed_weight_bytes(f->d_ff, f->d_model)) +
                     align256(packed_weight_bytes(f->d_model, f->d_ff));
  return per_layer * f->n_layers + align256(packed_weight_bytes(f->vocab, f->d_model));
}

extern "C" int dllm_pack_weights(dllm_ctx* c, void* stream, void* packed, size_t packed_bytes) {
  if (!c || !packed) return DLLM_EINVAL;
  const dllm_config& f = c->cfg;
  if (f.dtype != DLLM_BF16) return DLLM_ESHAPE;
  if (((uintptr_t)packed & 255) != 0) return DLLM_EINVAL;
  if (packed_bytes < dllm_packed_weight_bytes(&f)) return DLLM_ENOSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int dq = f.n_q_heads * f.head_dim, dkv = f.n_kv_heads * f.head_dim;
  if (!c->packed_layers) {
    c->packed_layers = (dllm_layer_w*)calloc(f.n_layers > 0 ? f.n_layers : 1, sizeof(dllm_layer_w));
    if (!c->packed_layers) return DLLM_ENOSPACE;
  }
  char* p = (char*)packed;
  auto pack = [&](const void* W, int N, int K, const void** dst) -> hipError_t {
    *dst = p;
    hipError_t e = launch_pack_weight(s, W, p, N, K);
    p += align256(packed_weight_bytes(N, K));
    return e;
  };
  for (int l = 0; l < f.n_layers; ++l) {
    const dllm_layer_w& L = c->layers[l];
    dllm_layer_w& P = c->packed_layers[l];
    TRY(pack(L.wq, dq, f.d_model, &P.wq), "pack wq");
    TRY(pack(L.wk, dkv, f.d_model, &P.wk), "pack wk");
    TRY(pack(L.wv, dkv, f.d_model, &P.wv), "pack wv");
    TRY(pack(L.wo, f.d_model, dq, &P.wo), "pack wo");
    TRY(pack(L.w_gate, f.d_ff, f.d_model, &P.w_gate), "pack w_gate");
    TRY(pack(L.w_up, f.d_ff, f.d_model, &P.w_up), "pack w_up");
    TRY(pack(L.w_down, f.d_model, f.d_ff, &P.w_down), "pack w_down");
  }
  TRY(pack(c->lm_head, f.vocab, f.d_model, &c->packed_lm_head), "pack lm_head");
  c->packed = (char*)packed;
  return DLLM_OK;
}

extern "C" void dllm_destroy(dllm_ctx* ctx) {
  if (!ctx) return;
  prof_free(ctx);
  free(ctx->packed_layers);
  free(ctx->layers);
  free(ctx);
}

extern "C" int dllm_set_kernel_mode(dllm_ctx* ctx, int mode) {
  if (!ctx || mode < 0 || mode > 1) return DLLM_EINVAL;
  ctx->kernel_mode = mode;
  return DLLM_OK;
}

extern "C" const char* dllm_strerror(int code) {
  switch (code) {
    case DLLM_OK: return "ok";
    case DLLM_EINVAL: return "invalid argument";
    case DLLM_ESHAPE: return "unsupported shape or above the configured maximum";
    case DLLM_ENOSPACE: return "workspace or KV pool too small";
    case DLLM_EHIP: return "HIP launch failed";
    default: return "unknown error";
  }
}

extern "C" const char* dllm_last_hip_error(const dllm_ctx* ctx) { return ctx ? ctx->hip_error : ""; }

#define WSP(c, field, type) ((type*)((c)->ws + (c)->map.field))

extern "C" int dllm_profile_enable(dllm_ctx* c, int on) {
  if (!c) return DLLM_EINVAL;
  if (!on) { c->prof_on = 0; return DLLM_OK; }
  if (!c->prof_ev) {
    const int cap = 8192;
    c->prof_ev = (hipEvent_t*)calloc(2 * cap, sizeof(hipEvent_t));
    c->prof_cls = (int*)calloc(cap, sizeof(int));
    c->prof_bytes = (double*)calloc(cap, sizeof(double));
    if (!c->prof_ev || !c->prof_cls || !c->prof_bytes) {
      free(c->prof_ev); free(c->prof_cls); free(c->prof_bytes);
      c->prof_ev = nullptr; c->prof_cls = nullptr; c->prof_bytes = nullptr;
      return DLLM_ENOSPACE;
    }
    for (int i = 0; i < 2 * cap; ++i) {
      hipError_t e = hipEventCreate(&c->prof_ev[i]);
      if (e != hipSuccess) {
        c->prof_cap = (i + 1) / 2;          // prof_free destroys 2 * prof_cap events: only those that exist
        for (int j = 2 * c->prof_cap; j < i; ++j) (void)hipEventDestroy(c->prof_ev[j]);
        prof_free(c);
        return hip_fail(c, e, "hipEventCreate");
      }
    }
    c->prof_cap = cap;
  }
  c->prof_n = 0;
  c->prof_on = 1;
  return DLLM_OK;
}

extern "C" int dllm_profile_read(dllm_ctx* c, void* stream, int cls, int32_t* n_launches, double* total_ms,
                                 double* total_bytes) {
  if (!c || !n_launches || !total_ms || !total_bytes) return DLLM_EINVAL;
  TRY(hipStreamSynchronize((hipStream_t)stream), "profile sync");
  int n = 0;
  double ms = 0.0, bytes = 0.0;
  for (int i = 0; i < c->prof_n; ++i) {
    if (c->prof_cls[i] != cls) continue;
    float t = 0.f;
    TRY(hipEventElapsedTime(&t, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]), "hipEventElapsedTime");
    ms += t; bytes += c->prof_bytes[i]; ++n;
  }
  *n_launches = n; *total_ms = ms; *total_bytes = bytes;
  return DLLM_OK;
}

// brackets one launch with events when profiling is on
struct ProfScope {
  dllm_ctx* c; hipStream_t s; int slot;
  ProfScope(dllm_ctx* c_, hipStream_t s_, int cls, double bytes) : c(c_), s(s_), slot(-1) {
    if (c->prof_on && c->prof_n < c->prof_cap) {
      slot = c->prof_n++;
      c->prof_cls[slot] = cls;
      c->prof_bytes[slot] = bytes;
      (void)hipEventRecord(c->prof_ev[2 * slot], s);
    }
  }
  ~ProfScope() { if (slot >= 0) (void)hipEventRecord(c->prof_ev[2 * slot + 1], s); }
};

// plain GEMM of the non-skinny path: matrix cores for bfloat16 (any M), scalar FMA otherwise
// norm_in: A is the output of an RMSNorm (bfloat16 models: x * gain, with the row factors in ws.rscale)
static hipError_t gemm_any(dllm_ctx* c, hipStream_t s, const void* A, const void* W, void* C, int M, int N, int K,
                           Epi epi, bool norm_in = false) {
  const float* rs = (norm_in && c->cfg.dtype == DLLM_BF16) ? (const float*)(c->ws + c->map.rscale) : nullptr;
  if (c->cfg.dtype == DLLM_BF16 && c->kernel_mode == 0 && N % 4 == 0 && K % 8 == 0)
    return launch_gemm_mfma(s, A, W, C, M, N, K, epi, rs, c->rows_dev);
  return launch_gemm_generic(c, s, A, W, C, M, N, K, epi, rs);
}

struct HeadOut {
  int32_t* cand;
  float* conf;
  float* entropy;
};

// The forward shared by all calls: embed, n_layers_run transformer layers over the rows of g,
// then optionally the residual stream, the raw logits or the fused confidence outputs.
static int run_forward_inner(dllm_ctx* c, hipStream_t s, const StepGeom& g, int n_layers_run, const HeadOut* head,
                             float* logits_out, float* hidden_out);

// the weight-streaming path: bfloat16 denoise steps of at most SK_MAX_ROWS rows
static bool skinny_path(const dllm_ctx* c, const StepGeom& g) {
  return mfma_supported(c) && g.Q > 0 && g.T <= SK_MAX_ROWS && attn_step_supported(c, g);
}

static int run_forward(dllm_ctx* c, hipStream_t s, const StepGeom& g0, int n_layers_run, const HeadOut* head,
                       float* logits_out, float* hidden_out) {
  // the first launches check the device-resident lengths against the host values that size the launches and leave
  // clamped copies in the workspace: every kernel after them addresses memory with those
  // (one launch together with the token map, the rotary table and the embedding on the weight-streaming path)
  const bool pro = skinny_path(c, g0);
  if (pro)
    TRY(launch_sk_prologue(c, s, g0, n_layers_run > 0 ? c->layers[0].attn_norm : c->final_norm,
                           head ? head->cand : nullptr, head ? head->conf : nullptr, head ? head->entropy : nullptr),
        "prologue");
  else TRY(launch_token_map(c, s, g0), "token_map");
  StepGeom g = g0;
  if (g.Q > 0) g.prefix_len = WSP(c, len_safe, int32_t);
  else g.cu_seqlens = WSP(c, len_safe, int32_t);
  if (g0.Q == 0 && g0.total_is_cap) {
    // the sequences may end before the buffer does: the row count is in the workspace for the GEMMs that can skip rows
    c->rows_dev = WSP(c, status, int32_t) + 2;
    const int rc = run_forward_inner(c, s, g, n_layers_run, head, logits_out, hidden_out);
    c->rows_dev = nullptr;
    return rc;
  }
  if (!g0.n_live) return run_forward_inner(c, s, g, n_layers_run, head, logits_out, hidden_out);
  // a step over the live sequences only: the valid rows per sequence (-1 for the sequences past the live count) and
  // the number of live rows are in the workspace as well
  g.q_valid = WSP(c, q_valid_eff, int32_t);
  c->rows_dev = WSP(c, status, int32_t) + 2;
  const int rc = run_forward_inner(c, s, g, n_layers_run, head, logits_out, hidden_out);
  c->rows_dev = nullptr;
  return rc;
}

static int run_forward_inner(dllm_ctx* c, hipStream_t s, const StepGeom& g, int n_layers_run, const HeadOut* head,
                             float* logits_out, float* hidden_out) {
  const dllm_config& f = c->cfg;
  const int T = g.T;
  const int dq = f.n_q_heads * f.head_dim, dkv = f.n_kv_heads * f.head_dim;
  // matrix-core kernels: bfloat16 denoise steps of at most SK_MAX_ROWS rows (weight streaming)
  // (their activation operands are kept in fragment order, which only these kernels write).  On this path no
  // RMSNorm is launched: the producer of the residual stream (embedding, output projection, down projection)
  // leaves x * gain of the next norm in fragment order plus partial sums of squares per row, and the consuming
  // GEMM applies the row's normalisation factor to its float accumulators.
  const bool sk = skinny_path(c, g);
  const bool big_mfma = f.dtype == DLLM_BF16 && c->kernel_mode == 0 && f.d_ff % 4 == 0 && f.vocab % 4 == 0;
  const int ss_groups = (f.d_model + 15) / 16;
  int n_ss = 1;      // partial sums of squares the current skinny-path GEMM input comes with
  if (!sk) {            // (on the weight-streaming path run_forward's prologue launch has done both)
    TRY(launch_embed(c, s, g), "embed");
    TRY(launch_rope_table(c, s, g), "rope_table");
  }
  int pending = 0;   // open residual sums (K splits of the last residual projection) not yet added to x
  for (int l = 0; l < n_layers_run; ++l) {
    const dllm_layer_w& L = c->layers[l];
    if (!sk) TRY(launch_rmsnorm(c, s, L.attn_norm, T, nullptr, nullptr, 0, pending), "rmsnorm");
    pending = 0;
    if (sk) {
      ProfScope p(c, s, 0, 2.0 * (dq + 2.0 * dkv) * f.d_model);
      TRY(launch_sk_qkv(c, s, g, l, attention_view(c, g, l), n_ss), "qkv");
    } else {
      ProfScope p(c, s, 0, 2.0 * T * (dq + 2.0 * dkv) * f.d_model);   // large path: work recorded in flops
      int n_part = 0;
      if (big_mfma) TRY(launch_gemm_qkv_split(c, s, c->ws + c->map.xn, L.wq, L.wk, L.wv, T, dq, dkv, f.d_model, &n_part), "wqkv");
      if (n_part > 0) {
        // q | k | v left as partial sums over K; the rotary kernel adds them
      } else if (big_mfma && f.d_model % 8 == 0 && dq % 4 == 0 && dkv % 4 == 0) {
        TRY(launch_gemm_qkv(s, c->ws + c->map.xn, L.wq, L.wk, L.wv, WSP(c, q32, float), WSP(c, k32, float),
                            c->ws + c->map.v, T, dq, dkv, f.d_model, WSP(c, rscale, float), c->rows_dev), "wqkv");
      } else {
        TRY(gemm_any(c, s, c->ws + c->map.xn, L.wq, c->ws + c->map.q32, T, dq, f.d_model, EPI_STORE_F32, true), "wq");
        TRY(gemm_any(c, s, c->ws + c->map.xn, L.wk, c->ws + c->map.k32, T, dkv, f.d_model, EPI_STORE_F32, true), "wk");
        TRY(gemm_any(c, s, c->ws + c->map.xn, L.wv, c->ws + c->map.v, T, dkv, f.d_model, EPI_STORE, true), "wv");
      }
      TRY(launch_rope_kv(c, s, g, l, n_part), "rope_kv");
    }
    {
      ProfScope p(c, s, 5, 2.0 * 2.0 * dkv * (double)g.max_kv * g.B);
      if (attn_step_supported(c, g)) TRY(launch_attn_step(c, s, g, attention_view(c, g, l), sk), "attention");
      else TRY(launch_attention_generic(c, s, g, l), "attention");
    }
    if (sk) {
      ProfScope p(c, s, 1, 2.0 * dq * f.d_model);
      TRY(launch_sk_resid(c, s, c->ws + c->map.o, c->packed_layers[l].wo, T, f.d_model, dq, L.mlp_norm), "wo");
      n_ss = ss_groups;
    } else {
      ProfScope p(c, s, 1, 2.0 * T * (double)dq * f.d_model);
      if (big_mfma && f.d_model % 4 == 0 && dq % 8 == 0)
        TRY(launch_gemm_resid_split(c, s, c->ws + c->map.o, L.wo, WSP(c, x, float), T, f.d_model, dq, &pending), "wo");
      else TRY(gemm_any(c, s, c->ws + c->map.o, L.wo, c->ws + c->map.x, T, f.d_model, dq, EPI_RESID), "wo");
    }
    if (!sk) TRY(launch_rmsnorm(c, s, L.mlp_norm, T, nullptr, nullptr, 0, pending), "rmsnorm");
    pending = 0;
    if (sk) {
      {
        ProfScope p(c, s, 2, 2.0 * 2.0 * f.d_ff * f.d_model);
        TRY(launch_sk_swiglu(c, s, l, T, n_ss), "swiglu");
      }
      ProfScope p(c, s, 3, 2.0 * f.d_ff * f.d_model);
      // the down projection prepares the input of whatever reads the residual stream next
      const void* gain_next = l + 1 < n_layers_run ? c->layers[l + 1].attn_norm : c->final_norm;
      TRY(launch_sk_resid(c, s, c->ws + c->map.h, c->packed_layers[l].w_down, T, f.d_model, f.d_ff, gain_next),
          "w_down");
    } else {
      if (big_mfma) {
        ProfScope p(c, s, 2, 2.0 * T * 2.0 * f.d_ff * f.d_model);
        // (the float gate buffer of the generic path is free here: scratch for the K-split tail tiles)
        TRY(launch_gemm_swiglu(s, c->ws + c->map.xn, L.w_gate, L.w_up, c->ws + c->map.h, T, f.d_ff, f.d_model,
                               WSP(c, rscale, float), c->rows_dev, WSP(c, g, float), c->map.g_bytes), "gate_up");
      } else {
        TRY(gemm_any(c, s, c->ws + c->map.xn, L.w_gate, c->ws + c->map.g, T, f.d_ff, f.d_model, EPI_STORE_F32, true), "w_gate");
        TRY(gemm_any(c, s, c->ws + c->map.xn, L.w_up, c->ws + c->map.u, T, f.d_ff, f.d_model, EPI_STORE_F32, true), "w_up");
        TRY(launch_swiglu(c, s, T), "swiglu");
      }
      ProfScope p(c, s, 3, 2.0 * T * (double)f.d_ff * f.d_model);
      if (big_mfma && f.d_model % 4 == 0 && f.d_ff % 8 == 0)
        TRY(launch_gemm_resid_split(c, s, c->ws + c->map.h, L.w_down, WSP(c, x, float), T, f.d_model, f.d_ff, &pending),
            "w_down");
      else TRY(gemm_any(c, s, c->ws + c->map.h, L.w_down, c->ws + c->map.x, T, f.d_model, f.d_ff, EPI_RESID), "w_down");
    }
  }
  if (hidden_out) {
    if (pending) { TRY(launch_fold_delta(c, s, T, pending, false), "fold_delta"); pending = 0; }
    TRY(launch_copy_f32(s, WSP(c, x, float), hidden_out, (size_t)T * f.d_model), "copy_hidden");
  }
  if (logits_out) {
    if (sk) {
      TRY(launch_sk_f32(c, s, c->ws + c->map.xn, c->packed_lm_head, logits_out, T, f.vocab, f.d_model, n_ss), "lm_head");
    } else {
      TRY(launch_rmsnorm(c, s, c->final_norm, T, nullptr, nullptr, 0, pending), "final_norm");
      pending = 0;
      TRY(gemm_any(c, s, c->ws + c->map.xn, c->lm_head, logits_out, T, f.vocab, f.d_model, EPI_STORE_F32, true), "lm_head");
    }
  }
  if (head) {
    const int max_rows = T < c->map.r_max ? T : (int)c->map.r_max;
    if (!sk) TRY(launch_mask_rows(c, s, g, head->cand, head->conf, head->entropy), "mask_rows");
    if (!sk) {
      TRY(launch_rmsnorm(c, s, c->final_norm, max_rows, WSP(c, rows, int32_t), WSP(c, status, int32_t) + 1, 0, pending),
          "final_norm");
      pending = 0;
    }
    int n_parts = c->map.n_vtiles;
    if (sk) {
      ProfScope p(c, s, 4, 2.0 * f.vocab * f.d_model);
      TRY(launch_sk_lmstats(c, s, T, n_ss, &n_parts), "lm_head");
    } else if (big_mfma) {
      ProfScope p(c, s, 4, 2.0 * max_rows * (double)f.vocab * f.d_model);   // upper bound: max_rows rows
      TRY(launch_gemm_lmstats(c, s, max_rows, &n_parts), "lm_head");
    } else TRY(launch_lm_head_generic(c, s, max_rows), "lm_head");
    TRY(launch_lm_merge(c, s, max_rows, n_parts, head->cand, head->conf, head->entropy, sk), "lm_merge");
  }
  return DLLM_OK;
}

static int check_step_args(dllm_ctx* c, int B, int Q, int max_prefix_len, const void* q_tokens,
                           const void* prefix_len, const void* block_table, bool padded = false) {
  if (!c || !q_tokens || !prefix_len || !block_table) return DLLM_EINVAL;
  if (B < 1 || Q < 1 || max_prefix_len < 0) return DLLM_EINVAL;
  if (B > c->cfg.max_batch || Q > c->cfg.max_q) return DLLM_ESHAPE;
  // with padding rows only the valid rows need pages (checked on the device, row by row)
  const int64_t reach = (int64_t)max_prefix_len + (padded ? 0 : Q);
  if (reach > (int64_t)c->cfg.max_pages_per_seq * c->cfg.page_tokens) return DLLM_ESHAPE;
  return DLLM_OK;
}

static StepGeom step_geom(int B, int Q, int max_prefix_len, const int32_t* q_tokens, const int32_t* prefix_len,
                          const int32_t* block_table) {
  StepGeom g;
  g.B = B; g.T = B * Q; g.Q = Q; g.max_kv = max_prefix_len + Q;
  g.tokens = q_tokens; g.prefix_len = prefix_len; g.cu_seqlens = nullptr; g.n_cache = nullptr;
  g.q_valid = nullptr;
  g.n_live = nullptr;
  g.block_table = block_table;
  return g;
}

extern "C" int dllm_denoise_step(dllm_ctx* c, void* stream, int B, int Q, int max_prefix_len,
                                 const int32_t* q_tokens, const int32_t* prefix_len, const int32_t* block_table,
                                 int32_t* cand_token, float* conf, float* entropy) {
  int rc = check_step_args(c, B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  if (rc != DLLM_OK) return rc;
  if (!cand_token || !conf) return DLLM_EINVAL;
  StepGeom g = step_geom(B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  HeadOut h{cand_token, conf, entropy};
  return run_forward(c, (hipStream_t)stream, g, c->cfg.n_layers, &h, nullptr, nullptr);
}

extern "C" int dllm_denoise_step_var(dllm_ctx* c, void* stream, int B, int Q, int max_prefix_len,
                                     const int32_t* q_tokens, const int32_t* prefix_len, const int32_t* q_valid,
                                     const int32_t* block_table, int32_t* cand_token, float* conf, float* entropy) {
  int rc = check_step_args(c, B, Q, max_prefix_len, q_tokens, prefix_len, block_table, true);
  if (rc != DLLM_OK) return rc;
  if (!cand_token || !conf || !q_valid) return DLLM_EINVAL;
  StepGeom g = step_geom(B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  g.q_valid = q_valid;
  HeadOut h{cand_token, conf, entropy};
  return run_forward(c, (hipStream_t)stream, g, c->cfg.n_layers, &h, nullptr, nullptr);
}

// ---- the denoise step for callers that cannot allocate ---------------------------------------------
// The intermediates of the step (everything the workspace of dllm_create holds) live in a file-scope
// device array instead.  Each GPU has its own copy of the array at its own address; the address is looked
// up once per device, with that device current, and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[DLLM_STATIC_SCRATCH_BYTES];
static constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];   // per device, nullptr until looked up

__global__ void k_or_status(int32_t* dst, const int32_t* src) {
  const int32_t v = src[0];
  if (v != 0) atomicOr(dst, v);
}

static int static_scratch(dllm_ctx* c, char** out) {
  int dev = -1;
  TRY(hipGetDevice(&dev), "hipGetDevice");
  if (dev < 0 || dev >= MAX_DEVICES) return DLLM_ESHAPE;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (!p || ((uintptr_t)p & 255) != 0) return DLLM_EINVAL;
    g_scratch_ptr[dev] = p;
  }
  *out = (char*)g_scratch_ptr[dev];
  return DLLM_OK;
}

extern "C" size_t dllm_static_scratch_bytes(void) { return (size_t)DLLM_STATIC_SCRATCH_BYTES; }

extern "C" int dllm_denoise_step_static(dllm_ctx* c, void* stream, int B, int Q, int max_prefix_len,
                                        const int32_t* q_tokens, const int32_t* prefix_len,
                                        const int32_t* block_table, int32_t* cand_token, float* conf,
                                        float* entropy) {
  int rc = check_step_args(c, B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  if (rc != DLLM_OK) return rc;
  if (!cand_token || !conf) return DLLM_EINVAL;
  if (c->map.total > (size_t)DLLM_STATIC_SCRATCH_BYTES) return DLLM_ENOSPACE;
  char* sp = nullptr;
  rc = static_scratch(c, &sp);
  if (rc != DLLM_OK) return rc;
  hipStream_t s = (hipStream_t)stream;
  char* const own = c->ws;
  int32_t* const own_status = WSP(c, status, int32_t);
  // the array keeps the previous call's contents: the status words are the only part a step reads before writing
  // (a fill kernel, not a memset node, so that the call can be captured into a graph)
  TRY(launch_set_i32(s, (int32_t*)(sp + c->map.status), 16, 0), "clear scratch status");
  StepGeom g = step_geom(B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  HeadOut h{cand_token, conf, entropy};
  c->ws = sp;
  rc = run_forward(c, s, g, c->cfg.n_layers, &h, nullptr, nullptr);
  c->ws = own;
  if (rc != DLLM_OK) return rc;
  k_or_status<<<1, 1, 0, s>>>(own_status, (const int32_t*)(sp + c->map.status));
  TRY(hipGetLastError(), "merge status");
  return DLLM_OK;
}

extern "C" int dllm_denoise_step_live(dllm_ctx* c, void* stream, int B, int Q, int max_prefix_len,
                                      const int32_t* q_tokens, const int32_t* prefix_len, const int32_t* q_valid,
                                      const int32_t* n_live, const int32_t* block_table, int32_t* cand_token,
                                      float* conf, float* entropy) {
  int rc = check_step_args(c, B, Q, max_prefix_len, q_tokens, prefix_len, block_table, true);
  if (rc != DLLM_OK) return rc;
  if (!cand_token || !conf || !n_live) return DLLM_EINVAL;
  StepGeom g = step_geom(B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  g.q_valid = q_valid;
  g.n_live = n_live;
  HeadOut h{cand_token, conf, entropy};
  return run_forward(c, (hipStream_t)stream, g, c->cfg.n_layers, &h, nullptr, nullptr);
}

static int check_rows_args(dllm_ctx* c, int B, int row_len, const void* index, const void* n_index, const void* src,
                           const void* dst) {
  if (!c || !index || !n_index || !src || !dst || src == dst) return DLLM_EINVAL;
  if (B < 1 || row_len < 1) return DLLM_EINVAL;
  if (B > (1 << 24) || row_len > (1 << 24)) return DLLM_ESHAPE;
  return DLLM_OK;
}

extern "C" int dllm_gather_rows(dllm_ctx* c, void* stream, int B, int row_len, const int32_t* index,
                                const int32_t* n_index, const int32_t* src, int32_t* dst, int32_t fill) {
  int rc = check_rows_args(c, B, row_len, index, n_index, src, dst);
  if (rc != DLLM_OK) return rc;
  TRY(launch_gather_rows((hipStream_t)stream, B, row_len, index, n_index, src, dst, fill, false), "gather_rows");
  return DLLM_OK;
}

extern "C" int dllm_scatter_rows(dllm_ctx* c, void* stream, int B, int row_len, const int32_t* index,
                                 const int32_t* n_index, const int32_t* src, int32_t* dst) {
  int rc = check_rows_args(c, B, row_len, index, n_index, src, dst);
  if (rc != DLLM_OK) return rc;
  TRY(launch_gather_rows((hipStream_t)stream, B, row_len, index, n_index, src, dst, 0, true), "scatter_rows");
  return DLLM_OK;
}

extern "C" int dllm_debug_logits(dllm_ctx* c, void* stream, int B, int Q, int max_prefix_len,
                                 const int32_t* q_tokens, const int32_t* prefix_len, const int32_t* block_table,
                                 float* logits) {
  int rc = check_step_args(c, B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  if (rc != DLLM_OK) return rc;
  if (!logits) return DLLM_EINVAL;
  StepGeom g = step_geom(B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  return run_forward(c, (hipStream_t)stream, g, c->cfg.n_layers, nullptr, logits, nullptr);
}

extern "C" int dllm_debug_hidden(dllm_ctx* c, void* stream, int B, int Q, int max_prefix_len,
                                 const int32_t* q_tokens, const int32_t* prefix_len, const int32_t* block_table,
                                 int n_layers_run, float* hidden) {
  int rc = check_step_args(c, B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  if (rc != DLLM_OK) return rc;
  if (!hidden || n_layers_run < 0 || n_layers_run > c->cfg.n_layers) return DLLM_EINVAL;
  StepGeom g = step_geom(B, Q, max_prefix_len, q_tokens, prefix_len, block_table);
  return run_forward(c, (hipStream_t)stream, g, n_layers_run, nullptr, nullptr, hidden);
}

static int packed_forward(dllm_ctx* c, void* stream, int B, int total_tokens, int max_seqlen,
                          const int32_t* tokens, const int32_t* cu_seqlens, const int32_t* n_cache,
                          const int32_t* block_table, const HeadOut* head, bool total_is_cap = false) {
  if (!c || !tokens || !cu_seqlens || !block_table) return DLLM_EINVAL;
  if (B < 1 || total_tokens < 1 || max_seqlen < 1 || max_seqlen > total_tokens) return DLLM_EINVAL;
  if (B > c->cfg.max_batch || total_tokens > c->cfg.max_tokens) return DLLM_ESHAPE;
  if (n_cache == nullptr && (int64_t)max_seqlen > (int64_t)c->cfg.max_pages_per_seq * c->cfg.page_tokens)
    return DLLM_ESHAPE;
  StepGeom g;
  g.B = B; g.T = total_tokens; g.Q = 0; g.max_kv = max_seqlen;
  g.tokens = tokens; g.prefix_len = nullptr; g.cu_seqlens = cu_seqlens; g.n_cache = n_cache;
  g.q_valid = nullptr;
  g.n_live = nullptr;
  g.block_table = block_table;
  g.total_is_cap = total_is_cap;
  return run_forward(c, (hipStream_t)stream, g, c->cfg.n_layers, head, nullptr, nullptr);
}

extern "C" int dllm_prefill_kv(dllm_ctx* c, void* stream, int B, int total_tokens, int max_seqlen,
                               const int32_t* tokens, const int32_t* cu_seqlens, const int32_t* n_cache,
                               const int32_t* block_table) {
  return packed_forward(c, stream, B, total_tokens, max_seqlen, tokens, cu_seqlens, n_cache, block_table, nullptr);
}

extern "C" int dllm_refresh_cache(dllm_ctx* c, void* stream, int B, int total_tokens, int max_seqlen,
                                  const int32_t* tokens, const int32_t* cu_seqlens, const int32_t* n_commit,
                                  const int32_t* block_table, int32_t* cand_token, float* conf, float* entropy) {
  if (cand_token == nullptr)
    return packed_forward(c, stream, B, total_tokens, max_seqlen, tokens, cu_seqlens, n_commit, block_table, nullptr);
  if (!conf || !n_commit) return DLLM_EINVAL;   // step outputs only make sense for rows past n_commit
  HeadOut h{cand_token, conf, entropy};
  return packed_forward(c, stream, B, total_tokens, max_seqlen, tokens, cu_seqlens, n_commit, block_table, &h);
}

extern "C" int dllm_refresh_cache_dev(dllm_ctx* c, void* stream, int B, int token_capacity, int max_seqlen,
                                      const int32_t* tokens, const int32_t* cu_seqlens, const int32_t* n_commit,
                                      const int32_t* block_table, int32_t* cand_token, float* conf, float* entropy) {
  if (!n_commit) return DLLM_EINVAL;
  if (cand_token == nullptr)
    return packed_forward(c, stream, B, token_capacity, max_seqlen, tokens, cu_seqlens, n_commit, block_table, nullptr, true);
  if (!conf) return DLLM_EINVAL;
  HeadOut h{cand_token, conf, entropy};
  return packed_forward(c, stream, B, token_capacity, max_seqlen, tokens, cu_seqlens, n_commit, block_table, &h, true);
}

extern "C" int dllm_unmask(dllm_ctx* c, void* stream, int B, int Q, int block_len, int32_t* q_tokens,
                           const int32_t* cand_token, const float* conf, float threshold, int min_unmask,
                           int32_t* n_unmasked, int32_t* n_remaining) {
  if (!c || !q_tokens || !cand_token || !conf) return DLLM_EINVAL;
  if (B < 1 || Q < 1 || block_len < 1 || min_unmask < 0 || Q % block_len != 0) return DLLM_EINVAL;
  if (threshold != threshold) return DLLM_EINVAL;
  if (block_len > 1024 || (int64_t)B * (Q / block_len) > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_unmask((hipStream_t)stream, B, Q, block_len, q_tokens, cand_token, conf, threshold, min_unmask,
                    c->cfg.mask_id, n_unmasked, n_remaining), "unmask");
  return DLLM_OK;
}

extern "C" int dllm_unmask_entropy(dllm_ctx* c, void* stream, int B, int Q, int block_len, int32_t* q_tokens,
                                   const int32_t* cand_token, const float* entropy, float theta, int min_unmask,
                                   int32_t* n_unmasked, int32_t* n_remaining) {
  if (!c || !q_tokens || !cand_token || !entropy) return DLLM_EINVAL;
  if (B < 1 || Q < 1 || block_len < 1 || min_unmask < 0 || Q % block_len != 0) return DLLM_EINVAL;
  if (theta != theta) return DLLM_EINVAL;
  if (block_len > 1024 || (int64_t)B * (Q / block_len) > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_unmask((hipStream_t)stream, B, Q, block_len, q_tokens, cand_token, entropy, theta, min_unmask,
                    c->cfg.mask_id, n_unmasked, n_remaining, true), "unmask_entropy");
  return DLLM_OK;
}

extern "C" int dllm_unmask_blocks(dllm_ctx* c, void* stream, int B, int Q, int block_len, int32_t* q_tokens,
                                  const int32_t* cand_token, const float* stat, float threshold, int by_entropy,
                                  const int32_t* floor, int32_t* n_unmasked, int32_t* n_remaining) {
  if (!c || !q_tokens || !cand_token || !stat || !floor) return DLLM_EINVAL;
  if (B < 1 || Q < 1 || block_len < 1 || Q % block_len != 0) return DLLM_EINVAL;
  if (threshold != threshold) return DLLM_EINVAL;
  if (block_len > 1024 || (int64_t)B * (Q / block_len) > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_unmask((hipStream_t)stream, B, Q, block_len, q_tokens, cand_token, stat, threshold, 0, c->cfg.mask_id,
                    n_unmasked, n_remaining, by_entropy != 0, floor), "unmask_blocks");
  return DLLM_OK;
}

extern "C" int dllm_fsm_update(dllm_ctx* c, void* stream, int B, int n_blocks, int block_len, const int32_t* gen_tokens,
                               int32_t* state, int32_t* counter, double add_at, double full_at, int delay,
                               int nocache_round, int32_t* floor_next, int32_t* summary) {
  if (!c || !gen_tokens || !state || !counter) return DLLM_EINVAL;
  if (B < 1 || n_blocks < 1 || block_len < 1 || delay < 0) return DLLM_EINVAL;
  if (!(add_at >= 0.0) || !(full_at >= 0.0)) return DLLM_EINVAL;
  if (n_blocks > DLLM_FSM_MAX_BLOCKS || B > (1 << 24) || block_len > (1 << 20)) return DLLM_ESHAPE;
  // the counts of unmasked positions from which "filled / block_len >= threshold" holds, in double
  int need_add = 0, need_full = 0;
  while (need_add <= block_len && (double)need_add / (double)block_len < add_at) ++need_add;
  while (need_full <= block_len && (double)need_full / (double)block_len < full_at) ++need_full;
  TRY(launch_fsm_update((hipStream_t)stream, B, n_blocks, block_len, gen_tokens, c->cfg.mask_id, state, counter,
                        need_add, need_full, delay, nocache_round < 0 ? -1 : (nocache_round != 0), floor_next, summary),
      "fsm_update");
  return DLLM_OK;
}

extern "C" int dllm_fsm_plan(dllm_ctx* c, void* stream, int B, int n_blocks, int block_len, const int32_t* state,
                             const int32_t* counter, const int32_t* base_len, int refresh_every, int32_t* rounds_since,
                             int32_t* nocache, int32_t* n_commit_next) {
  if (!c || !state || !counter || !rounds_since || !nocache || !n_commit_next) return DLLM_EINVAL;
  if (B < 1 || n_blocks < 1 || block_len < 1 || refresh_every < 0) return DLLM_EINVAL;
  if (n_blocks > DLLM_FSM_MAX_BLOCKS || B > (1 << 24) || block_len > (1 << 20)) return DLLM_ESHAPE;
  TRY(launch_fsm_plan((hipStream_t)stream, B, n_blocks, block_len, state, counter, base_len, refresh_every, rounds_since,
                      nocache, n_commit_next), "fsm_plan");
  return DLLM_OK;
}

extern "C" int dllm_fsm_window(dllm_ctx* c, void* stream, int B, int n_blocks, int block_len, int W,
                               const int32_t* gen_tokens, const int32_t* state, const int32_t* base_len,
                               int32_t pad_token, int32_t* win_tokens, int32_t* win_floor, int32_t* prefix_len,
                               int32_t* q_valid, int32_t* win_lo) {
  if (!c || !gen_tokens || !state || !base_len || !win_tokens || !win_floor || !prefix_len || !q_valid || !win_lo)
    return DLLM_EINVAL;
  if (B < 1 || n_blocks < 1 || block_len < 1 || W < 1) return DLLM_EINVAL;
  if (pad_token < 0 || pad_token >= c->cfg.vocab || pad_token == c->cfg.mask_id) return DLLM_EINVAL;
  if (n_blocks > DLLM_FSM_MAX_BLOCKS || B > (1 << 24) || (int64_t)W * block_len > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_fsm_window((hipStream_t)stream, B, n_blocks, block_len, W, gen_tokens, state, base_len, pad_token,
                        win_tokens, win_floor, prefix_len, q_valid, win_lo), "fsm_window");
  return DLLM_OK;
}

extern "C" int dllm_fsm_round_windows(dllm_ctx* c, void* stream, int B, int n_blocks, int block_len, int W,
                                      const int32_t* gen_tokens, const int32_t* state, const int32_t* base_len,
                                      const int32_t* nocache, int32_t pad_token, int32_t* win_tokens, int32_t* win_floor,
                                      int32_t* prefix_len, int32_t* q_valid, int32_t* q_valid_cached, int32_t* win_lo) {
  if (!c || !gen_tokens || !state || !base_len || !nocache || !win_tokens || !win_floor || !prefix_len || !q_valid ||
      !q_valid_cached || !win_lo)
    return DLLM_EINVAL;
  if (B < 1 || n_blocks < 1 || block_len < 1 || W < 1) return DLLM_EINVAL;
  if (pad_token < 0 || pad_token >= c->cfg.vocab || pad_token == c->cfg.mask_id) return DLLM_EINVAL;
  if (n_blocks > DLLM_FSM_MAX_BLOCKS || B > (1 << 24) || (int64_t)W * block_len > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_fsm_window((hipStream_t)stream, B, n_blocks, block_len, W, gen_tokens, state, base_len, pad_token,
                        win_tokens, win_floor, prefix_len, q_valid, win_lo, nocache, q_valid_cached), "fsm_round_windows");
  return DLLM_OK;
}

extern "C" int dllm_fsm_pack(dllm_ctx* c, void* stream, int B, int n_blocks, int block_len, int W, int max_prompt,
                             int token_capacity, int max_seqlen, const int32_t* prompt_tokens,
                             const int32_t* gen_tokens, const int32_t* state, const int32_t* base_len,
                             const int32_t* nocache, const int32_t* n_commit_plan, int32_t pad_token,
                             int32_t* tokens, int32_t* cu_seqlens, int32_t* n_commit) {
  if (!c || !prompt_tokens || !gen_tokens || !state || !base_len || !nocache || !n_commit_plan || !tokens ||
      !cu_seqlens || !n_commit)
    return DLLM_EINVAL;
  if (B < 1 || n_blocks < 1 || block_len < 1 || W < 1 || max_prompt < 1 || token_capacity < 1 || max_seqlen < 1)
    return DLLM_EINVAL;
  if (pad_token < 0 || pad_token >= c->cfg.vocab || pad_token == c->cfg.mask_id) return DLLM_EINVAL;
  if (n_blocks > DLLM_FSM_MAX_BLOCKS || B > (1 << 16) || (int64_t)n_blocks * block_len > (1 << 24) ||
      token_capacity > (1 << 28))
    return DLLM_ESHAPE;
  TRY(launch_fsm_pack((hipStream_t)stream, B, n_blocks, block_len, W, max_prompt, token_capacity, max_seqlen, state,
                      base_len, nocache, n_commit_plan, prompt_tokens, gen_tokens, pad_token, tokens, cu_seqlens,
                      n_commit, WSP(c, status, int32_t)), "fsm_pack");
  return DLLM_OK;
}

extern "C" int dllm_fsm_unpack(dllm_ctx* c, void* stream, int B, int Q, int token_capacity, const int32_t* cu_seqlens,
                               const int32_t* prefix_len, const int32_t* q_valid, const int32_t* nocache,
                               const int32_t* packed_cand, const float* packed_conf, const float* packed_entropy,
                               int32_t* cand_token, float* conf, float* entropy) {
  if (!c || !cu_seqlens || !prefix_len || !q_valid || !nocache || !packed_cand || !packed_conf || !cand_token || !conf)
    return DLLM_EINVAL;
  if (B < 1 || Q < 1 || token_capacity < 1) return DLLM_EINVAL;
  if (B > (1 << 24) || Q > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_fsm_unpack((hipStream_t)stream, B, Q, token_capacity, cu_seqlens, prefix_len, q_valid, nocache, packed_cand,
                        packed_conf, packed_entropy, cand_token, conf, entropy), "fsm_unpack");
  return DLLM_OK;
}

extern "C" int dllm_fsm_scatter(dllm_ctx* c, void* stream, int B, int n_blocks, int block_len, int W,
                                const int32_t* win_tokens, const int32_t* win_lo, const int32_t* q_valid,
                                int32_t* gen_tokens) {
  if (!c || !win_tokens || !win_lo || !q_valid || !gen_tokens) return DLLM_EINVAL;
  if (B < 1 || n_blocks < 1 || block_len < 1 || W < 1) return DLLM_EINVAL;
  if (n_blocks > DLLM_FSM_MAX_BLOCKS || B > (1 << 24) || (int64_t)W * block_len > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_fsm_scatter((hipStream_t)stream, B, n_blocks, block_len, W, win_tokens, win_lo, q_valid, gen_tokens),
      "fsm_scatter");
  return DLLM_OK;
}

extern "C" int dllm_unmask_traced(dllm_ctx* c, void* stream, int B, int Q, int block_len, int32_t* q_tokens,
                                  const int32_t* cand_token, const float* stat, float threshold, int by_entropy,
                                  int min_unmask, int32_t step_index, int32_t* order, int32_t* n_unmasked,
                                  int32_t* n_remaining) {
  if (!c || !q_tokens || !cand_token || !stat || !order) return DLLM_EINVAL;
  if (B < 1 || Q < 1 || block_len < 1 || min_unmask < 0 || Q % block_len != 0) return DLLM_EINVAL;
  if (threshold != threshold) return DLLM_EINVAL;
  if (block_len > 1024 || (int64_t)B * (Q / block_len) > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_unmask((hipStream_t)stream, B, Q, block_len, q_tokens, cand_token, stat, threshold, min_unmask,
                    c->cfg.mask_id, n_unmasked, n_remaining, by_entropy != 0, nullptr, order, step_index),
      "unmask_traced");
  return DLLM_OK;
}

extern "C" int dllm_noisy_sequence(dllm_ctx* c, void* stream, int B, int n, const int32_t* y, const int32_t* order,
                                   const int32_t* window_start, int k, double t, int32_t* out) {
  if (!c || !y || !order || !window_start || !out) return DLLM_EINVAL;
  if (B < 1 || n < 1 || k < 0 || !(t >= 0.0) || !(t <= 1.0)) return DLLM_EINVAL;
  if (B > 65535 || n > (1 << 28)) return DLLM_ESHAPE;
  const int kt = (int)ceil((double)k * t);
  TRY(launch_noisy_sequence((hipStream_t)stream, B, n, y, order, window_start, k, kt, c->cfg.mask_id, out),
      "noisy_sequence");
  return DLLM_OK;
}

extern "C" int dllm_eos_scan(dllm_ctx* c, void* stream, int B, int n, const int32_t* gen_tokens, int32_t eos_id,
                             int32_t* finished, int32_t* first_eos, int32_t* active_index, int32_t* n_active) {
  if (!c || !gen_tokens || !finished) return DLLM_EINVAL;
  if (B < 1 || n < 1 || (active_index == nullptr) != (n_active == nullptr)) return DLLM_EINVAL;
  if (eos_id < 0 || eos_id >= c->cfg.vocab || eos_id == c->cfg.mask_id) return DLLM_EINVAL;
  if (B > (1 << 24)) return DLLM_ESHAPE;
  TRY(launch_eos_scan((hipStream_t)stream, B, n, gen_tokens, eos_id, c->cfg.mask_id, finished, first_eos, active_index,
                      n_active), "eos_scan");
  return DLLM_OK;
}

extern "C" int dllm_probe_hbm_read(dllm_ctx* c, void* stream, const void* buf, size_t bytes, void* sink) {
  if (!c || !buf || !sink || bytes < 16 || ((uintptr_t)buf & 15) != 0) return DLLM_EINVAL;
  TRY(launch_probe_read((hipStream_t)stream, buf, bytes, sink), "probe_read");
  return DLLM_OK;
}

extern "C" int dllm_probe_mfma(dllm_ctx* c, void* stream, int iters, int random_bits, void* sink, double* flops) {
  if (!c || !sink || !flops || iters < 1 || iters > (1 << 24)) return DLLM_EINVAL;
  TRY(launch_probe_mfma((hipStream_t)stream, iters, random_bits != 0, sink, flops), "probe_mfma");
  return DLLM_OK;
}

extern "C" int dllm_reset_status(dllm_ctx* c, void* stream) {
  if (!c) return DLLM_EINVAL;
  TRY(launch_set_i32((hipStream_t)stream, WSP(c, status, int32_t), 16, 0), "reset_status");
  return DLLM_OK;
}

extern "C" int dllm_read_status(dllm_ctx* c, void* stream, int32_t* host_out) {
  if (!c || !host_out) return DLLM_EINVAL;
  TRY(hipMemcpyAsync(host_out, WSP(c, status, int32_t), sizeof(int32_t), hipMemcpyDeviceToHost, (hipStream_t)stream),
      "read_status");
  TRY(hipStreamSynchronize((hipStream_t)stream), "read_status sync");
  return DLLM_OK;
}
