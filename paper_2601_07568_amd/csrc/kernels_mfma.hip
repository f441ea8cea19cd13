// bfloat16 matrix-core (MFMA) kernels for gfx950.
//
// Skinny GEMM (at most 64 activation rows): the step is bound by streaming each weight once from
// HBM, so a workgroup owns a few 16-row tiles of the weight matrix for the whole K extent, its
// waves split K among themselves in interleaved 128-element blocks, every lane pulls 16-byte
// pieces of its weight row straight into registers (64 contiguous bytes per row and instruction,
// one block prefetched ahead), and the partial tiles are summed through LDS in a fixed order.
// The epilogue of the summed tile is the fusion point: residual add, rotary embedding + KV-cache
// write, SiLU*up, or the softmax statistics of the LM head (the logits never reach memory).
//
// v_mfma_f32_16x16x32_bf16 operand layout (lane l, c = l % 16, g = l / 16): A holds row c of a
// 16x32 tile, B holds column c of a 32x16 tile, each its 8 consecutive k-elements of group g;
// D holds column c, rows 4g..4g+3.  The k-order is immaterial as long as A and B agree, which is
// used here to give each lane contiguous bytes.
#include "common.h"
#include <math.h>
#include <string.h>

namespace dllm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                 0, 0);
}

enum SkEpi { SK_RESID = 0, SK_F32 = 1, SK_QKV = 2, SK_SWIGLU = 3, SK_LMSTATS = 4 };

struct SkArgs {
  const bf16_t* X;          // activations [M, K]
  const int32_t* m_dev;     // optional device row count (<= M)
  int M, K;
  const bf16_t* W0;         // main weight / Wq / W_gate / lm_head
  const bf16_t* W1;         // Wk / W_up
  const bf16_t* W2;         // Wv
  int N0, N1, N2;           // rows of W0, W1, W2
  float* out_f32;           // RESID: x [M, N0] (+=) ; F32: [M, N0]
  bf16_t* out_bf16;         // QKV: q [M, N0] ; SWIGLU: h [M, N0]
  // QKV
  int dh, n_q_wg, n_k_wg;   // head_dim, workgroups covering q, k
  const float* rope_cos;
  const float* rope_sin;
  const int32_t* tok_seq;
  const int32_t* tok_pos;
  bf16_t* pool_k;
  bf16_t* pool_v;
  KVView pool;
  int32_t* status;
  // LMSTATS
  float* part;              // [rows, n_parts, 4]
  int n_parts;
  int32_t mask_id;
};

constexpr int SK_KB = 128;  // k-elements per block: 4 matrix instructions deep

template <int NT, int MT>
struct SkFrag {
  u32x4 a[NT][4];
  u32x4 b[MT][4];
};

template <int NT, int MT, bool TAIL>
__device__ inline void sk_load(SkFrag<NT, MT>& f, const bf16_t* const (&wrow)[NT], const bf16_t* const (&xrow)[MT],
                               int kb, int g, int K) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int k = kb + j * 32;   // lane's element offset is k + g*8 (g*8 is folded into the row pointers)
    const bool ok = !TAIL || (k + g * 8 + 8 <= K);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (ok) f.a[t][j] = *(const u32x4*)(wrow[t] + k);
      else f.a[t][j] = u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      if (ok) f.b[t][j] = *(const u32x4*)(xrow[t] + k);
      else f.b[t][j] = u32x4{0, 0, 0, 0};
    }
  }
}

template <int NT, int MT>
__device__ inline void sk_mma(const SkFrag<NT, MT>& f, f32x4 (&acc)[NT][MT]) {
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int m = 0; m < MT; ++m) acc[t][m] = mfma16(f.a[t][j], f.b[m][j], acc[t][m]);
}

// first weight row of tile t of workgroup wg, and which matrix it belongs to
template <int NT, int EPI>
__device__ inline void sk_tile_rows(const SkArgs& a, int wg, const bf16_t* (&wbase)[NT], int (&row0)[NT],
                                    int (&nrows)[NT]) {
  if (EPI == SK_QKV) {
    const int half = a.dh >> 1, per_head = half / 16;
    if (wg < a.n_q_wg + a.n_k_wg) {
      const bool isq = wg < a.n_q_wg;
      const int lw = isq ? wg : wg - a.n_q_wg;
      const int h = lw / per_head, j0 = (lw - h * per_head) * 16;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        wbase[t] = isq ? a.W0 : a.W1;
        nrows[t] = isq ? a.N0 : a.N1;
        row0[t] = h * a.dh + j0 + t * half;
      }
    } else {
      const int lw = wg - a.n_q_wg - a.n_k_wg;
#pragma unroll
      for (int t = 0; t < NT; ++t) { wbase[t] = a.W2; nrows[t] = a.N2; row0[t] = lw * 16 * NT + t * 16; }
    }
  } else if (EPI == SK_SWIGLU) {
#pragma unroll
    for (int t = 0; t < NT; ++t) { wbase[t] = (t == 0) ? a.W0 : a.W1; nrows[t] = a.N0; row0[t] = wg * 16; }
  } else {
#pragma unroll
    for (int t = 0; t < NT; ++t) { wbase[t] = a.W0; nrows[t] = a.N0; row0[t] = wg * 16 * NT + t * 16; }
  }
}

template <int NT, int MT, int NW, int EPI>
__global__ __launch_bounds__(NW * 64) void k_skinny(const SkArgs a) {
  __shared__ float red[NW][NT][MT][4][64];
  __shared__ float lmst[EPI == SK_LMSTATS ? MT : 1][4][16][4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int wg = blockIdx.x;
  const int K = a.K;
  int M = a.M;
  if (a.m_dev) { const int md = *a.m_dev; M = md < M ? md : M; }
  if (M <= 0) return;

  const bf16_t* wbase[NT];
  int row0[NT], nrows[NT];
  sk_tile_rows<NT, EPI>(a, wg, wbase, row0, nrows);
  const bf16_t* wrow[NT];
  const bf16_t* xrow[MT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    int r = row0[t] + c;
    r = r < nrows[t] ? r : nrows[t] - 1;
    wrow[t] = wbase[t] + (int64_t)r * K + g * 8;
  }
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    int r = m * 16 + c;
    r = r < M ? r : M - 1;
    xrow[m] = a.X + (int64_t)r * K + g * 8;
  }

  f32x4 acc[NT][MT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[t][m] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int stride = NW * SK_KB;
  const int k_full = K / SK_KB * SK_KB;   // blocks below k_full need no tail guard
  SkFrag<NT, MT> f0, f1;
  int kb = w * SK_KB;
  if (kb < k_full) sk_load<NT, MT, false>(f0, wrow, xrow, kb, g, K);
  while (kb < k_full) {
    const int k1 = kb + stride;
    if (k1 < k_full) sk_load<NT, MT, false>(f1, wrow, xrow, k1, g, K);
    sk_mma<NT, MT>(f0, acc);
    if (k1 >= k_full) { kb = k1; break; }
    const int k2 = k1 + stride;
    if (k2 < k_full) sk_load<NT, MT, false>(f0, wrow, xrow, k2, g, K);
    sk_mma<NT, MT>(f1, acc);
    kb = k2;
  }
  if (k_full < K && w == (k_full / SK_KB) % NW) {   // ragged last block
    sk_load<NT, MT, true>(f0, wrow, xrow, k_full, g, K);
    sk_mma<NT, MT>(f0, acc);
  }

  // sum the waves' partial tiles in wave order
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int i = 0; i < 4; ++i) red[w][t][m][i][lane] = acc[t][m][i];
  __syncthreads();

  for (int item = tid; item < MT * 256; item += NW * 64) {
    const int m = item >> 8, i = (item >> 6) & 3, ln = item & 63;
    const int tok = m * 16 + (ln & 15);
    const int fr = 4 * (ln >> 4) + i;          // row inside the 16-row tile
    float val[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      float s = 0.f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) s += red[ww][t][m][i][ln];
      val[t] = s;
    }
    const bool tok_ok = tok < M;
    if (EPI == SK_RESID || EPI == SK_F32) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int n = row0[t] + fr;
        if (tok_ok && n < a.N0) {
          float* p = a.out_f32 + (int64_t)tok * a.N0 + n;
          if (EPI == SK_RESID) *p += val[t]; else *p = val[t];
        }
      }
    } else if (EPI == SK_SWIGLU) {
      const int n = row0[0] + fr;
      if (tok_ok && n < a.N0) {
        const float gt = val[0];
        a.out_bf16[(int64_t)tok * a.N0 + n] = f32_to_bf16(gt / (1.0f + expf(-gt)) * val[NT - 1]);
      }
    } else if (EPI == SK_QKV) {
      if (tok_ok) {
        if (wg < a.n_q_wg + a.n_k_wg) {
          const bool isq = wg < a.n_q_wg;
          const int half = a.dh >> 1;
          const int hj = row0[0] + fr;                 // h*dh + j, j < half
          const int h = hj / a.dh, j = hj - h * a.dh;
          const float cs = a.rope_cos[(int64_t)tok * half + j], sn = a.rope_sin[(int64_t)tok * half + j];
          const float v0 = val[0], v1 = val[NT - 1];
          const bf16_t r0 = f32_to_bf16(v0 * cs - v1 * sn), r1 = f32_to_bf16(v1 * cs + v0 * sn);
          if (isq) {
            a.out_bf16[(int64_t)tok * a.N0 + hj] = r0;
            a.out_bf16[(int64_t)tok * a.N0 + hj + half] = r1;
          } else {
            int64_t ko, vo;
            int vs;
            if (kv_locate(a.pool, a.tok_seq[tok], a.tok_pos[tok], h, ko, vo, vs)) {
              a.pool_k[ko + j] = r0;
              a.pool_k[ko + j + half] = r1;
            } else atomicOr(a.status, DLLM_STATUS_BAD_PAGE);
          }
        } else {
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const int n = row0[t] + fr;
            if (n < a.N2) {
              const int h = n / a.dh, ch = n - h * a.dh;
              int64_t ko, vo;
              int vs;
              if (kv_locate(a.pool, a.tok_seq[tok], a.tok_pos[tok], h, ko, vo, vs))
                a.pool_v[vo + (int64_t)ch * vs] = f32_to_bf16(val[t]);
            }
          }
        }
      }
    } else if (EPI == SK_LMSTATS) {
      RowStat st;
      st.init();
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int n = row0[t] + fr;
        if (n < a.N0 && n != a.mask_id) st.merge(val[t], n, 1.0f, val[t]);
      }
      // same token: lanes ln, ln^16, ln^32, ln^48 of this wave, then the four values of i
#pragma unroll
      for (int o = 16; o < 64; o <<= 1) {
        const float m2 = __shfl_xor(st.m, o, 64), s2 = __shfl_xor(st.s, o, 64), t2 = __shfl_xor(st.t, o, 64);
        const int i2 = __shfl_xor(st.idx, o, 64);
        st.merge(m2, i2, s2, t2);
      }
      if ((ln >> 4) == 0) {
        float* p = &lmst[m][i][ln & 15][0];
        p[0] = st.m; p[1] = __int_as_float(st.idx); p[2] = st.s; p[3] = st.t;
      }
    }
  }
  if (EPI == SK_LMSTATS) {
    __syncthreads();
    if (tid < MT * 16) {
      const int m = tid >> 4, cc = tid & 15, tok = m * 16 + cc;
      if (tok < M) {
        RowStat st;
        st.init();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float* p = &lmst[m][i][cc][0];
          st.merge(p[0], __float_as_int(p[1]), p[2], p[3]);
        }
        float* o = a.part + ((int64_t)tok * a.n_parts + wg) * 4;
        o[0] = st.m; o[1] = __int_as_float(st.idx); o[2] = st.s; o[3] = st.t;
      }
    }
  }
}

template <int NT, int NW, int EPI>
static hipError_t sk_launch_mt(hipStream_t s, const SkArgs& a, int grid) {
  const int mt = (a.M + 15) / 16;
  switch (mt) {
    case 1: k_skinny<NT, 1, NW, EPI><<<grid, NW * 64, 0, s>>>(a); break;
    case 2: k_skinny<NT, 2, NW, EPI><<<grid, NW * 64, 0, s>>>(a); break;
    case 3: k_skinny<NT, 3, NW, EPI><<<grid, NW * 64, 0, s>>>(a); break;
    case 4: k_skinny<NT, 4, NW, EPI><<<grid, NW * 64, 0, s>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

#define WSM(c, field, type) ((type*)((c)->ws + (c)->map.field))

bool mfma_supported(const dllm_ctx* c) {
  const dllm_config& f = c->cfg;
  return f.dtype == DLLM_BF16 && c->kernel_mode == 0 && f.d_model % 8 == 0 && f.d_ff % 8 == 0 &&
         (f.head_dim == 64 || f.head_dim == 128);
}

static SkArgs sk_base(const void* X, int M, int K) {
  SkArgs a;
  memset(&a, 0, sizeof(a));
  a.X = (const bf16_t*)X;
  a.M = M;
  a.K = K;
  return a;
}

// x[M,N] += A[M,K] * W[N,K]^T
hipError_t launch_sk_resid(dllm_ctx* c, hipStream_t s, const void* A, const void* W, float* x, int M, int N, int K) {
  SkArgs a = sk_base(A, M, K);
  a.W0 = (const bf16_t*)W;
  a.N0 = N;
  a.out_f32 = x;
  return sk_launch_mt<1, 8, SK_RESID>(s, a, (N + 15) / 16);
}

// out[M,N] = A[M,K] * W[N,K]^T in float (debug logits)
hipError_t launch_sk_f32(dllm_ctx* c, hipStream_t s, const void* A, const void* W, float* out, int M, int N, int K) {
  SkArgs a = sk_base(A, M, K);
  a.W0 = (const bf16_t*)W;
  a.N0 = N;
  a.out_f32 = out;
  return sk_launch_mt<4, 4, SK_F32>(s, a, (N + 63) / 64);
}

// fused q/k/v projection of a denoise step: rotary embedding on q and k, q to the workspace,
// k and v into the in-flight pages of the pool
hipError_t launch_sk_qkv(dllm_ctx* c, hipStream_t s, const StepGeom& g, int layer, const KVView& pool) {
  const dllm_config& f = c->cfg;
  const dllm_layer_w& L = c->layers[layer];
  SkArgs a = sk_base(c->ws + c->map.xn, g.T, f.d_model);
  a.W0 = (const bf16_t*)L.wq; a.W1 = (const bf16_t*)L.wk; a.W2 = (const bf16_t*)L.wv;
  a.N0 = f.n_q_heads * f.head_dim; a.N1 = a.N2 = f.n_kv_heads * f.head_dim;
  a.out_bf16 = WSM(c, q, bf16_t);
  a.dh = f.head_dim;
  const int per_head = f.head_dim / 2 / 16;
  a.n_q_wg = f.n_q_heads * per_head;
  a.n_k_wg = f.n_kv_heads * per_head;
  a.rope_cos = WSM(c, rope_cos, float); a.rope_sin = WSM(c, rope_sin, float);
  a.tok_seq = WSM(c, tok_seq, int32_t); a.tok_pos = WSM(c, tok_pos, int32_t);
  a.pool_k = (bf16_t*)pool.k; a.pool_v = (bf16_t*)pool.v; a.pool = pool;
  a.status = WSM(c, status, int32_t);
  const int n_v_wg = (a.N2 + 31) / 32;
  return sk_launch_mt<2, 8, SK_QKV>(s, a, a.n_q_wg + a.n_k_wg + n_v_wg);
}

// h[M,F] = silu(xn Wg^T) * (xn Wu^T)
hipError_t launch_sk_swiglu(dllm_ctx* c, hipStream_t s, int layer, int M) {
  const dllm_config& f = c->cfg;
  const dllm_layer_w& L = c->layers[layer];
  SkArgs a = sk_base(c->ws + c->map.xn, M, f.d_model);
  a.W0 = (const bf16_t*)L.w_gate; a.W1 = (const bf16_t*)L.w_up;
  a.N0 = f.d_ff;
  a.out_bf16 = WSM(c, h, bf16_t);
  return sk_launch_mt<2, 8, SK_SWIGLU>(s, a, (f.d_ff + 15) / 16);
}

// LM head on the compacted rows (ws.xn) -> per-64-column softmax statistics
hipError_t launch_sk_lmstats(dllm_ctx* c, hipStream_t s, int max_rows, int* n_parts_out) {
  const dllm_config& f = c->cfg;
  SkArgs a = sk_base(c->ws + c->map.xn, max_rows, f.d_model);
  a.m_dev = WSM(c, status, int32_t) + 1;
  a.W0 = (const bf16_t*)c->lm_head;
  a.N0 = f.vocab;
  a.part = WSM(c, lm_part, float);
  a.n_parts = (f.vocab + 63) / 64;
  a.mask_id = f.mask_id;
  *n_parts_out = a.n_parts;
  return sk_launch_mt<4, 4, SK_LMSTATS>(s, a, a.n_parts);
}

}  // namespace dllm
