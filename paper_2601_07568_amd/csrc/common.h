// Shared declarations of the denoise-step library: context, workspace map, KV addressing,
// bf16 helpers, and the internal launch functions that api.hip chains together.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/dllm.h"

namespace dllm {

typedef uint16_t bf16_t;  // bfloat16 bit pattern

__host__ __device__ inline float bf16_to_f32(bf16_t b) {
  union { uint32_t u; float f; } c;
  c.u = ((uint32_t)b) << 16;
  return c.f;
}
// round to nearest, ties to even; NaN stays NaN
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// Fragment order of a bfloat16 activation matrix [rows, K] that feeds the weight-streaming GEMM:
// element (row, k) lives at frag_offset(row, k, mt), mt = 16-row tiles of the matrix.  The 16-byte
// unit of (128-element block kb, instruction j, tile m, lane g*16 + c) holds row m*16 + c,
// k = kb*128 + j*32 + g*8 .. +7, so that every operand fetch of a wave is one contiguous KiB.
__host__ __device__ inline int64_t frag_offset(int row, int k, int mt) {
  const int kb = k >> 7, j = (k >> 5) & 3, g = (k >> 3) & 3;
  return ((((int64_t)kb * 4 + j) * mt + (row >> 4)) * 64 + g * 16 + (row & 15)) * 8 + (k & 7);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  __device__ static inline float load(const float* p) { return *p; }
  __device__ static inline void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  __device__ static inline float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static inline void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Where the keys/values of a forward live.
// Paged (table != nullptr): position j of sequence b is in page table[b*max_pages + j/page_tokens],
// slot j%page_tokens.  Per layer the K slab is [n_pages][n_kv_heads][page_tokens][head_dim] and the
// V slab is stored transposed, [n_pages][n_kv_heads][head_dim][page_tokens], so that the keys of
// one channel are contiguous (the layout the P*V matrix instruction wants for its operand).
// Packed (table == nullptr): the scratch of a no-cache forward, K [n_kv_heads][tpad][head_dim] and
// V [n_kv_heads][head_dim][tpad]; sequence b starts at column cu_pad[b] (a multiple of 32).
struct KVView {
  const void* k;
  const void* v;
  const int32_t* table;   // nullptr = packed
  const int32_t* cu_pad;  // packed only
  int32_t page_tokens, max_pages, n_pages, n_kv_heads, head_dim, tpad;
};

// Element offsets of (sequence b, position pos, kv head h): k_off addresses channel 0 of the K
// row; channel c of V is at v_off + c * v_stride.  Returns false if the position is not
// addressable (beyond the block table, or a table entry outside the pool).
__device__ inline bool kv_locate(const KVView& kv, int b, int pos, int h, int64_t& k_off, int64_t& v_off,
                                 int& v_stride) {
  if (kv.table == nullptr) {
    const int64_t col = (int64_t)kv.cu_pad[b] + pos;
    k_off = ((int64_t)h * kv.tpad + col) * kv.head_dim;
    v_off = (int64_t)h * kv.head_dim * kv.tpad + col;
    v_stride = kv.tpad;
    return true;
  }
  const int pi = pos / kv.page_tokens;
  if (pos < 0 || pi >= kv.max_pages) return false;
  const int page = kv.table[(int64_t)b * kv.max_pages + pi];
  if (page < 0 || page >= kv.n_pages) return false;
  const int slot = pos - pi * kv.page_tokens;
  const int64_t ph = (int64_t)page * kv.n_kv_heads + h;
  k_off = (ph * kv.page_tokens + slot) * kv.head_dim;
  v_off = ph * kv.head_dim * kv.page_tokens + slot;
  v_stride = kv.page_tokens;
  return true;
}

#define DEV_INF (__builtin_inff())

// Softmax statistics of a run of logits in ascending column order.
struct RowStat {
  float m, s, t;  // running max, sum exp(z-m), sum exp(z-m)*z
  int idx;
  __device__ inline void init() { m = -DEV_INF; s = 0.f; t = 0.f; idx = 0x7fffffff; }
  __device__ inline void push(float z, int col) {
    if (z > m) {
      float a = expf(m - z);   // exp(-inf) = 0 on the first value
      s = s * a + 1.0f;
      t = t * a + z;
      m = z;
      idx = col;
    } else {
      float e = expf(z - m);
      s += e;
      t = fmaf(e, z, t);
    }
  }
  // merge with another run; on equal maxima the lower column wins
  __device__ inline void merge(float m2, int i2, float s2, float t2) {
    if (!(s2 > 0.f) && !(s2 != s2)) return;   // empty run
    if (!(s > 0.f) && !(s != s)) { m = m2; idx = i2; s = s2; t = t2; return; }
    if (m2 > m || (m2 == m && i2 < idx)) {
      float a = expf(m - m2);
      s = s * a + s2;
      t = t * a + t2;
      m = m2;
      idx = i2;
    } else {
      float a = expf(m2 - m);
      s = fmaf(s2, a, s);
      t = fmaf(t2, a, t);
    }
  }
};

// Workspace map (byte offsets from the workspace base), fixed at dllm_create.
struct Workspace {
  size_t status;       // int32[16]: [0] status bits, [1] number of LM-head rows
  size_t x;            // float [Tmax, d]          residual stream
  size_t xn;           // T     [Tmax, d]          normalised activations (GEMM input)
  size_t q32;          // float [Tmax, Hq*dh]      q projection before the rotary embedding
  size_t k32;          // float [Tmax, Hkv*dh]     k projection before the rotary embedding
  size_t q;            // T     [Tmax, Hq*dh]      rotated q
  size_t v;            // T     [Tmax, Hkv*dh]     v projection, token-major
  size_t kpack;        // T     [Hkv, tpad, dh]    rotated K of a no-cache forward
  size_t vpack;        // T     [Hkv, dh, tpad]    V of a no-cache forward, transposed
  size_t cu_pad;       // int32 [max_batch + 1]    padded column offset of each packed sequence
  size_t o;            // T     [Tmax, Hq*dh]      attention output
  size_t g;            // float [Tmax, F]          gate pre-activation (generic path)
  size_t u;            // float [Tmax, F]          up projection (generic path)
  size_t h;            // T     [Tmax, F]          silu(g)*u
  size_t rope_cos;     // float [Tmax, dh/2]
  size_t rope_sin;     // float [Tmax, dh/2]
  size_t tok_seq;      // int32 [Tmax]             sequence of each packed token
  size_t tok_pos;      // int32 [Tmax]             position of each token in its sequence
  size_t rows;         // int32 [Rmax]             compacted list of LM-head rows
  size_t lm_part;      // float [Rmax, n_vtiles, 4] per-tile (max, argmax, sumexp, sum e*z)
  size_t attn_part;    // float [attn_rows, dh] partial outputs, then [attn_rows, 2] (max, sum) of split-KV units
  int64_t attn_rows;   // capacity in (token, head, unit) rows
  size_t len_safe;     // int32 [max_batch + 1]         checked prefix lengths (step) or sequence offsets (packed forward)
  size_t q_valid_eff;  // int32 [max_batch]             valid rows per sequence of a step with a live count (-1: not live)
  size_t rscale;       // float [Tmax]                  row normalisation factors of the current GEMM input (bfloat16 models)
  size_t ss;           // float [64][d/16 rounded up to 4]   partial sums of squares of the rows of the skinny path's GEMM input
  size_t delta;        // float open residual sums of K-split residual projections: [LG_MAX_DELTA][lg_delta_rows, d]
  int64_t delta_stride;
  int64_t lg_delta_rows, lg_delta_stride;   // large path: rows the buffer covers (0 = none), floats per split
  size_t qkvp;         // float [LG_QKV_SPLITS][lg_delta_rows, dq + 2 dkv]: K-split partial sums of the fused q/k/v product
  int64_t qkvp_stride;
  int64_t qkvp_rows;   // rows a single (unsplit) product may have
  size_t scratch;      // general scratch for fast kernels (split-K partials)
  size_t total;
  int64_t t_max, r_max, t_step, tpad;
  int32_t n_vtiles, max_splits;
  size_t scratch_bytes;
  size_t g_bytes;      // size of the g region (bfloat16 models on the matrix-core path use it for K-split tail tiles)
};

}  // namespace dllm

struct dllm_ctx {
  dllm_config cfg;
  dllm_layer_w* layers;      // host copy
  const void *tok_emb, *final_norm, *lm_head;
  // weights in fragment order (dllm_pack_weights); nullptr until packed
  char* packed;
  dllm_layer_w* packed_layers;   // host array; norm gains are not packed and left null
  const void* packed_lm_head;
  char* kv_pool;
  char* ws;
  dllm::Workspace map;
  int kernel_mode;
  const int32_t* rows_dev;   // during a step with a live count: device count of rows the large GEMMs compute; else nullptr
  char hip_error[256];
  // per-kernel event timing (dllm_profile_*)
  int prof_on, prof_n, prof_cap;
  hipEvent_t* prof_ev;       // 2 * prof_cap events
  int* prof_cls;
  double* prof_bytes;
};

namespace dllm {

inline size_t elem_size(const dllm_config& c) { return c.dtype == DLLM_BF16 ? 2 : 4; }
inline size_t kv_slab_elems(const dllm_config& c) {
  return (size_t)c.n_pages * c.n_kv_heads * c.page_tokens * c.head_dim;
}
constexpr int LM_TILE_N = 512;      // vocabulary columns per LM-head partial
constexpr int ATTN_MAX_SPLITS = 64;

// ---- launchers implemented in kernels_generic.hip (any shape, both dtypes) -------------------
struct StepGeom {           // which tokens a forward runs over
  int B, T;                 // sequences, total rows
  int Q;                    // rows per sequence (step) or 0 (packed, ragged)
  int max_kv;               // upper bound of keys any row attends to (launch sizing)
  const int32_t* tokens;    // dev [T]
  const int32_t* prefix_len;   // dev [B] (step) or nullptr
  const int32_t* q_valid;      // dev [B] or nullptr (step): rows of a sequence past q_valid[b] are padding - they are
                               // no keys for the other rows and get no LM-head row
  const int32_t* n_live;       // dev [1] or nullptr (step): sequences b >= n_live[0] are not part of the call (no
                               // attention, no cache write, no LM-head row; GEMM rows past the live ones are skipped)
  const int32_t* cu_seqlens;   // dev [B+1] (packed) or nullptr
  bool total_is_cap = false;   // packed: T is the capacity of the token buffer, the device-resident total may be smaller
  const int32_t* n_cache;      // dev [B] or nullptr (packed: how many positions go to the pool)
  const int32_t* block_table;  // dev [B, max_pages]
};

hipError_t launch_token_map(dllm_ctx* c, hipStream_t s, const StepGeom& g);
// steps of at most 64 rows on the matrix-core path: length checks, token map, rotary table, embedding and (cand != nullptr)
// the LM head's row list with the fixed outputs of the rows that are not masked, in one launch
hipError_t launch_sk_prologue(dllm_ctx* c, hipStream_t s, const StepGeom& g, const void* gain, int32_t* cand,
                              float* conf, float* entropy);
hipError_t launch_embed(dllm_ctx* c, hipStream_t s, const StepGeom& g);
hipError_t launch_rope_table(dllm_ctx* c, hipStream_t s, const StepGeom& g);
// out[T or n_rows, d] = rmsnorm(x[row]) * gain; rows == nullptr: identity row map, n = T
// frag_mt > 0: write in fragment order for frag_mt 16-row tiles (bfloat16 only)
// n_delta > 0 (fragment path only): first add the open residual sums delta_0 .. to x
hipError_t launch_rmsnorm(dllm_ctx* c, hipStream_t s, const void* gain, int T, const int32_t* rows,
                          const int32_t* n_rows_dev, int frag_mt, int n_delta);
hipError_t launch_fold_delta(dllm_ctx* c, hipStream_t s, int T, int n_delta, bool frag_path);
constexpr int LG_QKV_SPLITS = 3;       // large path: most K splits of the fused q/k/v product
constexpr int LG_MAX_DELTA = 3;        // large path: a residual projection is split over K at most 4 ways
constexpr int LG_DELTA_ROWS = 2048;    // ... and only when the token count leaves the chip underfilled
hipError_t launch_sk_resid(dllm_ctx* c, hipStream_t s, const void* A, const void* W, int M, int N, int K,
                           const void* gain_next);
enum Epi { EPI_STORE = 0, EPI_STORE_F32 = 1, EPI_RESID = 2 };
// C[M,N] (=, or +=) A[M,K] * W[N,K]^T ; A and W of the model dtype
hipError_t launch_gemm_generic(dllm_ctx* c, hipStream_t s, const void* A, const void* W, void* C,
                               int M, int N, int K, Epi epi, const float* rscale = nullptr);
hipError_t launch_rope_kv(dllm_ctx* c, hipStream_t s, const StepGeom& g, int layer, int n_part = 0);
hipError_t launch_swiglu(dllm_ctx* c, hipStream_t s, int T);
hipError_t launch_attention_generic(dllm_ctx* c, hipStream_t s, const StepGeom& g, int layer);
hipError_t launch_mask_rows(dllm_ctx* c, hipStream_t s, const StepGeom& g, int32_t* cand, float* conf,
                            float* entropy);
hipError_t launch_lm_head_generic(dllm_ctx* c, hipStream_t s, int max_rows);
// by_token: the partial statistics of compacted row r are stored at row rows[r] (the LM head ran on every row)
hipError_t launch_lm_merge(dllm_ctx* c, hipStream_t s, int max_rows, int n_parts, int32_t* cand, float* conf,
                           float* entropy, bool by_token = false);
hipError_t launch_unmask(hipStream_t s, int B, int Q, int block_len, int32_t* q_tokens,
                         const int32_t* cand, const float* conf, float thr, int min_unmask,
                         int32_t mask_id, int32_t* n_unmasked, int32_t* n_remaining, bool low_first = false, const int32_t* floors = nullptr,
                         int32_t* order = nullptr, int32_t step_index = 0);
hipError_t launch_fsm_window(hipStream_t s, int B, int n_blocks, int block_len, int W, const int32_t* gen,
                             const int32_t* state, const int32_t* base_len, int32_t pad_token, int32_t* win_tokens,
                             int32_t* win_floor, int32_t* prefix_len, int32_t* q_valid, int32_t* win_lo,
                             const int32_t* nocache = nullptr, int32_t* q_valid_cached = nullptr);
hipError_t launch_fsm_pack(hipStream_t s, int B, int n_blocks, int block_len, int W, int max_prompt, int cap,
                           int max_seqlen, const int32_t* state, const int32_t* base_len, const int32_t* nocache,
                           const int32_t* n_commit_plan, const int32_t* prompt, const int32_t* gen, int32_t pad_token,
                           int32_t* tokens, int32_t* cu, int32_t* n_commit, int32_t* status);
hipError_t launch_fsm_unpack(hipStream_t s, int B, int Q, int cap, const int32_t* cu, const int32_t* prefix_len,
                             const int32_t* q_valid, const int32_t* nocache, const int32_t* src_cand,
                             const float* src_conf, const float* src_ent, int32_t* cand, float* conf, float* ent);
hipError_t launch_fsm_scatter(hipStream_t s, int B, int n_blocks, int block_len, int W, const int32_t* win_tokens,
                              const int32_t* win_lo, const int32_t* q_valid, int32_t* gen);
hipError_t launch_noisy_sequence(hipStream_t s, int B, int n, const int32_t* y, const int32_t* order, const int32_t* s_dev,
                                 int k, int kt, int32_t mask_id, int32_t* out);
hipError_t launch_eos_scan(hipStream_t s, int B, int n, const int32_t* gen, int32_t eos_id, int32_t mask_id,
                           int32_t* finished, int32_t* first_eos, int32_t* active_index, int32_t* n_active);
hipError_t launch_fsm_update(hipStream_t s, int B, int n_blocks, int block_len, const int32_t* gen, int32_t mask_id,
                             int32_t* state, int32_t* counter, int need_add, int need_full, int delay, int nocache_round,
                             int32_t* floor_next, int32_t* summary);
hipError_t launch_fsm_plan(hipStream_t s, int B, int n_blocks, int block_len, const int32_t* state,
                           const int32_t* counter, const int32_t* base_len, int refresh_every, int32_t* rounds_since,
                           int32_t* nocache, int32_t* n_commit_next);
hipError_t launch_copy_f32(hipStream_t s, const float* src, float* dst, size_t n);
hipError_t launch_gather_rows(hipStream_t s, int B, int row_len, const int32_t* index, const int32_t* n_index,
                              const int32_t* src, int32_t* dst, int32_t fill, bool scatter);

// ---- launchers implemented in kernels_skinny.hip / kernels_attention.hip / kernels_gemm.hip (bf16, matrix cores) --
bool mfma_supported(const dllm_ctx* c);
size_t packed_weight_bytes(int N, int K);
hipError_t launch_pack_weight(hipStream_t s, const void* W, void* P, int N, int K);
constexpr int SK_MAX_ROWS = 64;   // the skinny (weight-streaming) kernels take at most this many rows
KVView attention_view(dllm_ctx* c, const StepGeom& g, int layer);
// n_ss: partial sums of squares per row the GEMM input comes with (1 after the embedding, d_model / 64 after a
// residual projection)
hipError_t launch_sk_f32(dllm_ctx* c, hipStream_t s, const void* A, const void* W, float* out, int M, int N, int K,
                         int n_ss);
hipError_t launch_sk_qkv(dllm_ctx* c, hipStream_t s, const StepGeom& g, int layer, const KVView& pool, int n_ss);
hipError_t launch_sk_swiglu(dllm_ctx* c, hipStream_t s, int layer, int M, int n_ss);
hipError_t launch_sk_lmstats(dllm_ctx* c, hipStream_t s, int T, int n_ss, int* n_parts_out);
hipError_t launch_gemm_mfma(hipStream_t s, const void* A, const void* W, void* C, int M, int N, int K, Epi epi,
                            const float* rscale = nullptr, const int32_t* m_dev = nullptr);
hipError_t init_attn_kernels();   // once per process (raises a kernel's LDS limit)
hipError_t init_gemm_t256();   // once per process, before the first large GEMM (raises a kernel's LDS limit)
hipError_t launch_gemm_resid_split(dllm_ctx* c, hipStream_t s, const void* A, const void* W, float* x, int M, int N, int K,
                                   int* n_delta);
hipError_t launch_gemm_qkv_split(dllm_ctx* c, hipStream_t s, const void* A, const void* Wq, const void* Wk, const void* Wv,
                                 int M, int dq, int dkv, int K, int* n_part);
hipError_t launch_gemm_qkv(hipStream_t s, const void* A, const void* Wq, const void* Wk, const void* Wv, float* q32,
                           float* k32, void* v, int M, int dq, int dkv, int K, const float* rscale,
                           const int32_t* m_dev);
// tail / tail_bytes: optional float scratch for the K-split tail tiles of the 256-row kernel (nullptr: none)
hipError_t launch_gemm_swiglu(hipStream_t s, const void* A, const void* Wg, const void* Wu, void* H, int M, int F,
                              int K, const float* rscale, const int32_t* m_dev, float* tail = nullptr,
                              size_t tail_bytes = 0);
hipError_t launch_gemm_lmstats(dllm_ctx* c, hipStream_t s, int max_rows, int* n_parts_out);
hipError_t launch_probe_read(hipStream_t s, const void* buf, size_t bytes, void* sink);
hipError_t launch_probe_mfma(hipStream_t s, int iters, int random_bits, void* sink, double* flops);
bool attn_step_supported(const dllm_ctx* c, const StepGeom& g);
hipError_t launch_attn_step(dllm_ctx* c, hipStream_t s, const StepGeom& g, const KVView& kv, bool frag_out);

}  // namespace dllm
