// bfloat16 matrix-core (MFMA) kernels for gfx950: the weight-streaming GEMMs of a denoise step.
//
// Skinny GEMM (at most 64 activation rows): the step is bound by streaming each weight once from
// HBM, so a workgroup owns a few 16-row tiles of the weight matrix for the whole K extent, its
// waves split K among themselves in interleaved 128-element blocks, every lane pulls 16-byte
// pieces of its weight row straight into registers (64 contiguous bytes per row and instruction,
// one block prefetched ahead), and the partial tiles are summed through LDS in a fixed order.
// The epilogue of the summed tile is the fusion point: residual add, rotary embedding + KV-cache
// write, SiLU*up, or the softmax statistics of the LM head (the logits never reach memory).
//
#include "mfma_common.h"

namespace dllm {

enum SkEpi { SK_F32 = 1, SK_QKV = 2, SK_SWIGLU = 3, SK_LMSTATS = 4, SK_DELTA = 5 };

struct SkArgs {
  const bf16_t* X;          // activations [M, K]
  const int32_t* m_dev;     // optional device row count (<= M)
  int M, K;
  const bf16_t* W0;         // main weight / Wq / W_gate / lm_head   (all in packed fragment order)
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
  // DELTA: grid.y splits K; split y stores its partial product to out_f32 + y * delta_stride, [M, N0];
  // the consumer of the residual stream adds the splits up in order
  int sps;                  // stages per split (0: no split)
  int64_t delta_stride;
  // LMSTATS
  float* part;              // [rows, n_parts, 4]
  int n_parts;
  int32_t mask_id;
};

constexpr int SK_KB = 128;  // k-elements per block: 4 matrix instructions deep
constexpr int SK_NW = 8;    // waves of a workgroup (they split K among themselves)

// One pipeline stage: JB matrix-instruction steps (JB*32 k-elements) of NT weight tiles and MT
// activation tiles.
template <int NT, int MT, int JB>
struct SkFrag {
  u32x4 a[NT][JB];
  u32x4 b[MT][JB];
};

// Both operands are in fragment order: step u (32 k-elements) of weight tile t is the KiB at
// wt[t] + u*64 units, of activation tile m the KiB at xf + (u*MT + m)*64 units (lane offset folded
// into the pointers), so every load instruction of the wave is contiguous.
template <int NT, int MT, int JB, bool TAIL>
__device__ inline void sk_load(SkFrag<NT, MT, JB>& f, const u32x4* const (&wt)[NT], const u32x4* xf, int stage, int g,
                               int K) {
#pragma unroll
  for (int j = 0; j < JB; ++j) {
    const int u = stage * JB + j;
#pragma unroll
    for (int t = 0; t < NT; ++t) f.a[t][j] = wt[t][u * 64];   // packed weights are zero beyond K
    // the activation buffer is not: beyond K it holds whatever was there, and 0 * NaN is NaN
    const bool ok = !TAIL || (u * 32 + g * 8 + 8 <= K);
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      if (ok) f.b[t][j] = xf[(u * MT + t) * 64];
      else f.b[t][j] = u32x4{0, 0, 0, 0};
    }
  }
}

template <int NT, int MT, int JB>
__device__ inline void sk_mma(const SkFrag<NT, MT, JB>& f, f32x4 (&acc)[NT][MT]) {
#pragma unroll
  for (int j = 0; j < JB; ++j)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int m = 0; m < MT; ++m) acc[t][m] = mfma16(f.a[t][j], f.b[m][j], acc[t][m]);
}

// first weight row of tile t of workgroup wg, and which matrix it belongs to
template <int NT, int EPI>
__device__ inline void sk_tile_rows(const SkArgs& a, int wg, const bf16_t* (&wbase)[NT], int (&row0)[NT],
                                    int (&nrows)[NT]) {
  if constexpr (EPI == SK_QKV) {
    // NT == 3: tiles 0 and 1 are the two halves of rotary pair-tile wg (rows h*dh + j0 .. and the same
    // + dh/2) of Wq or Wk, tile 2 is 16-row tile wg of Wv: pair tiles and value tiles are handed out
    // together so that the grid is max(pair tiles, value tiles) equal workgroups
    const int half = a.dh >> 1, per_head = half / 16;
    const int n_pairs = a.n_q_wg + a.n_k_wg;
    const int pw = wg < n_pairs ? wg : n_pairs - 1;            // clamped: the result is dropped
    const bool isq = pw < a.n_q_wg;
    const int lw = isq ? pw : pw - a.n_q_wg;
    const int h = lw / per_head, j0 = (lw - h * per_head) * 16;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      wbase[t] = isq ? a.W0 : a.W1;
      nrows[t] = isq ? a.N0 : a.N1;
      row0[t] = h * a.dh + j0 + t * half;
    }
    wbase[NT - 1] = a.W2;
    nrows[NT - 1] = a.N2;
    row0[NT - 1] = wg * 16;                                    // beyond N2: clamped by the caller, dropped below
  } else if constexpr (EPI == SK_SWIGLU) {
    // NT = 2*P: tiles 0..P-1 are P consecutive 16-row tiles of the gate matrix, tiles P..2P-1 the same rows of up
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      wbase[t] = (t < NT / 2) ? a.W0 : a.W1;
      nrows[t] = a.N0;
      row0[t] = (wg * (NT / 2) + (t % (NT / 2))) * 16;
    }
  } else {
#pragma unroll
    for (int t = 0; t < NT; ++t) { wbase[t] = a.W0; nrows[t] = a.N0; row0[t] = wg * 16 * NT + t * 16; }
  }
}

// (second launch bound: at least 4 waves per SIMD, i.e. two 8-wave workgroups per CU, so that one
// workgroup's prologue and reduction overlap the other's streaming)
template <int NT, int MT, int NW, int EPI>
__global__ __launch_bounds__(NW * 64, (NT + MT == 4 && NW == 8) ? 4 : ((NW == 4 && MT >= 3) ? 2 : 1)) void k_skinny(const SkArgs a) {
  // weight bytes in flight per wave: two stages of NT*JB KiB; with three or four activation tiles the
  // shorter stage keeps the kernel at two workgroups per CU
  constexpr int JB = (NT == 1) ? 4 : ((MT >= 3 || EPI == SK_DELTA) ? 1 : 2);
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
  // packed weights: the 16-row tile rt of a matrix with kpb 128-element blocks starts at unit
  // rt * kpb * 256; inside, (block, j, lane) is unit (block*4 + j)*64 + lane: one contiguous stream
  const int kpb = (K + SK_KB - 1) / SK_KB;
  const u32x4* wt[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    int rt = row0[t] >> 4;
    const int rt_max = (nrows[t] + 15) / 16 - 1;
    rt = rt < rt_max ? rt : rt_max;
    wt[t] = (const u32x4*)wbase[t] + (int64_t)rt * kpb * 256 + lane;
  }
  const u32x4* xf = (const u32x4*)a.X + lane;   // rows >= M of the last tile hold stale data: their columns are dropped

  f32x4 acc[NT][MT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[t][m] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Software pipeline over this wave's stages (w, w+NW, ...): two stages are in flight while a third
  // is multiplied.  No load sits inside a branch of the steady-state loop (a branch around a load
  // makes the compiler wait for every outstanding load at the join); the drain is straight-line code.
  constexpr int SKB = JB * 32;                        // k-elements per stage
  const int n_full = K / SKB;                         // stages that need no tail guard
  const int ws = __builtin_amdgcn_readfirstlane(w);   // wave index as a scalar
  const int s_lo = a.sps > 0 ? (int)blockIdx.y * a.sps : 0;          // this workgroup's range of stages
  const int s_hi = a.sps > 0 ? (s_lo + a.sps < n_full ? s_lo + a.sps : n_full) : n_full;
  const int n_loc = s_hi > s_lo ? s_hi - s_lo : 0;
  const int n_w = n_loc > ws ? (n_loc - ws + NW - 1) / NW : 0;
#define SK_LD(F, I) sk_load<NT, MT, JB, false>(F, wt, xf, s_lo + ws + (I) * NW, g, K)
#define SK_MM(F) sk_mma<NT, MT, JB>(F, acc)
  if (n_w == 1) {
    SkFrag<NT, MT, JB> f0;
    SK_LD(f0, 0);
    SK_MM(f0);
  } else if (n_w > 1) {
    SkFrag<NT, MT, JB> f0, f1, f2;
    SK_LD(f0, 0);
    SK_LD(f1, 1);
    int i = 0;
    while (i + 4 < n_w) {          // stages i .. i+4 exist
      SK_LD(f2, i + 2); SK_MM(f0);
      SK_LD(f0, i + 3); SK_MM(f1);
      SK_LD(f1, i + 4); SK_MM(f2);
      i += 3;
    }
    switch (n_w - i) {             // 2, 3 or 4 stages left; f0 = stage i, f1 = stage i+1 in flight
      case 2: SK_MM(f0); SK_MM(f1); break;
      case 3: SK_LD(f2, i + 2); SK_MM(f0); SK_MM(f1); SK_MM(f2); break;
      default: SK_LD(f2, i + 2); SK_MM(f0); SK_LD(f0, i + 3); SK_MM(f1); SK_MM(f2); SK_MM(f0); break;
    }
  }
#undef SK_LD
#undef SK_MM
  if (n_full * SKB < K && blockIdx.y == gridDim.y - 1 && ws == n_loc % NW) {   // ragged last stage
    SkFrag<NT, MT, JB> ft;
    sk_load<NT, MT, JB, true>(ft, wt, xf, n_full, g, K);
    sk_mma<NT, MT, JB>(ft, acc);
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
    if constexpr (EPI == SK_F32 || EPI == SK_DELTA) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int n = row0[t] + fr;
        if (tok_ok && n < a.N0) {
          float* p = a.out_f32 + (int64_t)tok * a.N0 + n;
          if (EPI == SK_DELTA) p[(int64_t)blockIdx.y * a.delta_stride] = val[t];
          else *p = val[t];
        }
      }
    } else if constexpr (EPI == SK_SWIGLU) {
#pragma unroll
      for (int t = 0; t < NT / 2; ++t) {
        const int n = row0[t] + fr;
        if (tok_ok && n < a.N0) {
          const float gt = val[t];
          a.out_bf16[frag_offset(tok, n, MT)] = f32_to_bf16(gt / (1.0f + expf(-gt)) * val[t + NT / 2]);
        }
      }
    } else if constexpr (EPI == SK_QKV) {
      if (tok_ok) {
        if (wg < a.n_q_wg + a.n_k_wg) {
          const bool isq = wg < a.n_q_wg;
          const int half = a.dh >> 1;
          const int hj = row0[0] + fr;                 // h*dh + j, j < half
          const int h = hj / a.dh, j = hj - h * a.dh;
          const float cs = a.rope_cos[(int64_t)tok * half + j], sn = a.rope_sin[(int64_t)tok * half + j];
          const float v0 = val[0], v1 = val[1];
          const bf16_t r0 = f32_to_bf16(v0 * cs - v1 * sn), r1 = f32_to_bf16(v1 * cs + v0 * sn);
          if (isq) {
            a.out_bf16[(int64_t)tok * a.N0 + hj] = r0;
            a.out_bf16[(int64_t)tok * a.N0 + hj + half] = r1;
          } else {
            int64_t ko, vo;
            int vs;
            if (a.tok_pos[tok] < 0) {
              // a padding row: nothing of it is cached
            } else if (kv_locate(a.pool, a.tok_seq[tok], a.tok_pos[tok], h, ko, vo, vs)) {
              a.pool_k[ko + j] = r0;
              a.pool_k[ko + j + half] = r1;
            } else atomicOr(a.status, DLLM_STATUS_BAD_PAGE);
          }
        }
        const int n = row0[NT - 1] + fr;               // value row
        if (n < a.N2) {
          const int h = n / a.dh, ch = n - h * a.dh;
          int64_t ko, vo;
          int vs;
          if (a.tok_pos[tok] >= 0 && kv_locate(a.pool, a.tok_seq[tok], a.tok_pos[tok], h, ko, vo, vs))
            a.pool_v[vo + (int64_t)ch * vs] = f32_to_bf16(val[NT - 1]);
        }
      }
    } else if constexpr (EPI == SK_LMSTATS) {
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

// ---- weight packing ---------------------------------------------------------------------------
// [N, K] row-major -> fragment order, rows padded to 16 and K to 128 with zeros.  Unit (16 bytes)
// index ((rt * kpb + kb) * 4 + j) * 64 + g*16 + c holds row rt*16 + c, k = kb*128 + j*32 + g*8 .. +7.
__global__ void k_pack_weight(const bf16_t* __restrict__ W, u32x4* __restrict__ P, int N, int K, int64_t n_units) {
  const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= n_units) return;
  const int kpb = (K + SK_KB - 1) / SK_KB;
  const int lane = (int)(u & 63), j = (int)((u >> 6) & 3);
  const int64_t t = u >> 8;
  const int kb = (int)(t % kpb), rt = (int)(t / kpb);
  const int r = rt * 16 + (lane & 15), k = kb * SK_KB + j * 32 + (lane >> 4) * 8;
  u32x4 v = u32x4{0, 0, 0, 0};
  if (r < N && k + 8 <= K) v = *(const u32x4*)(W + (int64_t)r * K + k);
  P[u] = v;
}

size_t packed_weight_bytes(int N, int K) {
  return (size_t)((N + 15) / 16) * ((K + SK_KB - 1) / SK_KB) * 256 * 16;
}

hipError_t launch_pack_weight(hipStream_t s, const void* W, void* P, int N, int K) {
  const int64_t n_units = (int64_t)(packed_weight_bytes(N, K) / 16);
  k_pack_weight<<<(unsigned)((n_units + 255) / 256), 256, 0, s>>>((const bf16_t*)W, (u32x4*)P, N, K, n_units);
  return hipGetLastError();
}


bool mfma_supported(const dllm_ctx* c) {
  const dllm_config& f = c->cfg;
  return f.dtype == DLLM_BF16 && c->kernel_mode == 0 && c->packed != nullptr && f.d_model <= 16384 && f.d_model % 8 == 0 && f.d_ff % 8 == 0 &&
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

// Residual projection with the sum over K left open: split y of K writes A*W^T restricted to its
// K range into delta + y*delta_stride ([M, N] float); the next RMSNorm adds x + delta_0 + delta_1 ..
// in that order.  With K split across workgroups a workgroup can own 64 weight rows instead of 16
// (the activation operand is re-read a quarter as often) and small N still fills the chip.
// Returns the number of splits through n_splits.
hipError_t launch_sk_delta(dllm_ctx* c, hipStream_t s, const void* A, const void* W, float* delta,
                           int64_t delta_stride, int max_splits, int M, int N, int K, int* n_splits) {
  SkArgs a = sk_base(A, M, K);
  a.W0 = (const bf16_t*)W;   // packed
  a.N0 = N;
  a.out_f32 = delta;
  a.delta_stride = delta_stride;
  const int groups = (N + 63) / 64;
  const int n_full = K / 32;                       // the kernel's stages: one 32-element step each (JB = 1)
  int ks = (256 + groups - 1) / groups;
  if (ks > max_splits) ks = max_splits;
  if (ks > n_full / (2 * SK_NW)) ks = n_full / (2 * SK_NW);   // at least two stages per wave
  if (ks < 1) ks = 1;
  int sps = (n_full + ks - 1) / ks;
  sps = (sps + SK_NW - 1) / SK_NW * SK_NW;         // every wave the same number of stages
  if (sps < SK_NW) sps = SK_NW;
  ks = n_full > 0 ? (n_full + sps - 1) / sps : 1;
  a.sps = sps;
  *n_splits = ks;
  const int mt = (M + 15) / 16;
  dim3 grid(groups, ks);
  switch (mt) {
    case 1: k_skinny<4, 1, SK_NW, SK_DELTA><<<grid, SK_NW * 64, 0, s>>>(a); break;
    case 2: k_skinny<4, 2, SK_NW, SK_DELTA><<<grid, SK_NW * 64, 0, s>>>(a); break;
    case 3: k_skinny<4, 3, SK_NW, SK_DELTA><<<grid, SK_NW * 64, 0, s>>>(a); break;
    case 4: k_skinny<4, 4, SK_NW, SK_DELTA><<<grid, SK_NW * 64, 0, s>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
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
  const dllm_layer_w& P = c->packed_layers[layer];
  a.W0 = (const bf16_t*)P.wq; a.W1 = (const bf16_t*)P.wk; a.W2 = (const bf16_t*)P.wv;
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
  const int n_pairs = a.n_q_wg + a.n_k_wg, n_vt = (a.N2 + 15) / 16;
  return sk_launch_mt<3, SK_NW, SK_QKV>(s, a, n_pairs > n_vt ? n_pairs : n_vt);
}

// h[M,F] = silu(xn Wg^T) * (xn Wu^T), written in fragment order for the down projection
hipError_t launch_sk_swiglu(dllm_ctx* c, hipStream_t s, int layer, int M) {
  const dllm_config& f = c->cfg;
  const dllm_layer_w& L = c->layers[layer];
  SkArgs a = sk_base(c->ws + c->map.xn, M, f.d_model);
  const dllm_layer_w& P = c->packed_layers[layer];
  a.W0 = (const bf16_t*)P.w_gate; a.W1 = (const bf16_t*)P.w_up;
  a.N0 = f.d_ff;
  a.out_bf16 = WSM(c, h, bf16_t);
  // (three tile pairs per workgroup -- 256 equal workgroups at F = 12288 -- measured no faster than one)
  return sk_launch_mt<2, SK_NW, SK_SWIGLU>(s, a, (f.d_ff + 15) / 16);
}

// LM head on the compacted rows (ws.xn) -> per-64-column softmax statistics
hipError_t launch_sk_lmstats(dllm_ctx* c, hipStream_t s, int max_rows, int* n_parts_out) {
  const dllm_config& f = c->cfg;
  SkArgs a = sk_base(c->ws + c->map.xn, max_rows, f.d_model);
  a.m_dev = WSM(c, status, int32_t) + 1;
  a.W0 = (const bf16_t*)c->packed_lm_head;
  a.N0 = f.vocab;
  a.part = WSM(c, lm_part, float);
  a.n_parts = (f.vocab + 63) / 64;
  a.mask_id = f.mask_id;
  *n_parts_out = a.n_parts;
  return sk_launch_mt<4, 4, SK_LMSTATS>(s, a, a.n_parts);
}

}  // namespace dllm
