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
#include <stdlib.h>

namespace dllm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                 0, 0);
}

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
__global__ __launch_bounds__(NW * 64, (NT + MT == 4 && NW == 8) ? 4 : 1) void k_skinny(const SkArgs a) {
  constexpr int JB = (NT == 1) ? 4 : 2;   // weight bytes in flight per wave: two stages of NT*JB KiB
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

#define WSM(c, field, type) ((type*)((c)->ws + (c)->map.field))

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
  const int n_full = K / 64;                       // stages of JB = 2 steps
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

// ==========================================================================================
// Block-query attention of a denoise step over the paged pool, register-direct: no LDS.
//
// One wave owns 16*QT query rows of one (sequence, kv head) -- with grouped-query attention the
// rows are (head-in-group, token) pairs -- and walks 32-key blocks.  S^T = K Q^T is computed with
// K rows as the A operand; A-row rho of tile t is given key 8*(rho/4) + rho%4 + 4t of the block,
// so that the accumulator layout (column = query, rows 4g..4g+3) leaves lane group g holding
// exactly keys 8g..8g+7 of each query: the B operand of O^T = V^T P^T without any shuffle.  V is
// stored transposed in the pool, so the A operand of that product is a 16-byte load as well.
// Softmax statistics of a query live in the lanes that hold its column.  Several units (waves)
// may split the keys of one row group; each writes an unnormalised partial (m, l, O) and
// k_attn_combine merges them.
struct AttnArgs {
  const bf16_t* q;          // [T, Hq, DH] rotated
  const int32_t* prefix_len;  // denoise step: keys = prefix_len[b] + Q (or + q_valid[b])
  const int32_t* q_valid;     // denoise step, optional: rows past q_valid[b] are padding and no keys
  const int32_t* cu;          // no-cache forward (Q == 0): sequence b is rows cu[b] .. cu[b+1], keys = its length
  bf16_t* o;                // output when n_units == 1 (row-major, or fragment order if out_mt > 0)
  int out_mt;
  KVView kv;
  int Q, Hq, Hkv, B;
  int n_units;              // key-splitting units per row group (gridDim.x * waves along keys)
  int kspl;                 // units (waves along the keys) inside a workgroup; their partials are merged in LDS
  int n_parts;              // partials per row = workgroups along the keys
  int n_rg_wg;              // row groups per workgroup
  int pt_shift;             // log2(page_tokens) if that is a power of two (0 for the packed scratch), else -1
  float scale_log2;         // log2(e) / sqrt(DH)
  float* part_o;            // [T*Hq, n_units, DH]
  float* part_ml;           // [T*Hq, n_units, 2]
  int32_t* status;
};

// two floats -> packed bfloat16 pair (round to nearest even, in hardware)
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}

// Online softmax of one 32-key block for QT query tiles; the lane holds raw scores of keys
// k0 + 8g + 4tt + i.  Updates the running maximum (in log2 units), the lane's share of the
// denominator and rescales the accumulators only when some maximum of the wave moved.
// Probabilities enter the second product as a bfloat16 pair hi + lo (two instructions): a
// single rounding of p would be the largest error of the whole attention and would flip the
// rounding of a good fraction of the stored outputs.
template <int DT, int QT>
__device__ __forceinline__ void attn_softmax_block(f32x4 (&s)[2][QT], int k0, int kv_len, int g, float scale_log2,
                                                   float (&m_run)[QT], float (&l_run)[QT], f32x4 (&oacc)[DT][QT],
                                                   u32x4 (&pf)[QT], u32x4 (&pl)[QT]) {
  if (k0 + 32 > kv_len) {                               // only a sequence's last block has keys to mask
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (k0 + 8 * g + 4 * tt + i >= kv_len) s[tt][t][i] = -DEV_INF;
  }
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float mx = fmaxf(fmaxf(fmaxf(s[0][t][0], s[0][t][1]), fmaxf(s[0][t][2], s[0][t][3])),
                     fmaxf(fmaxf(s[1][t][0], s[1][t][1]), fmaxf(s[1][t][2], s[1][t][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run[t], mx * scale_log2);   // finite: every block has at least one valid key
    if (__builtin_amdgcn_ballot_w64(m_new > m_run[t]) != 0) {
      const float alpha = __builtin_amdgcn_exp2f(m_run[t] - m_new);   // exp2(-inf) = 0 on the first block
      l_run[t] *= alpha;
#pragma unroll
      for (int d = 0; d < DT; ++d) oacc[d][t] = oacc[d][t] * alpha;
      m_run[t] = m_new;
    }
    float p[8], ps = 0.f;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float e = __builtin_amdgcn_exp2f(fmaf(s[tt][t][i], scale_log2, -m_new));
        p[tt * 4 + i] = e;
        ps += e;
      }
    l_run[t] += ps;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t h = pack_bf16x2(p[2 * e], p[2 * e + 1]);
      pf[t][e] = h;
      pl[t][e] = pack_bf16x2(p[2 * e] - __uint_as_float(h << 16), p[2 * e + 1] - __uint_as_float(h & 0xffff0000u));
    }
  }
}

template <int DH, int QT>
__global__ __launch_bounds__(256) void k_attn_step(const AttnArgs a) {
  constexpr int KK = DH / 32;   // k-steps of Q K^T
  constexpr int DT = DH / 16;   // 16-row tiles of O^T
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int rg = blockIdx.y * a.n_rg_wg + (w % a.n_rg_wg);
  const int unit = blockIdx.x * a.kspl + (w / a.n_rg_wg);
  extern __shared__ __attribute__((aligned(16))) unsigned char attn_smem[];
  const int b = blockIdx.z / a.Hkv, kvh = blockIdx.z - b * a.Hkv;
  const int G = a.Hq / a.Hkv;
  const bool paged = a.Q > 0;
  const int row_base = paged ? b * a.Q : a.cu[b];               // first row of the sequence in q / o
  const int n_q = paged ? a.Q : a.cu[b + 1] - a.cu[b];          // its query rows
  const int R = n_q * G;
  if (rg * 16 * QT >= R) return;
  const int kv_len = paged ? a.prefix_len[b] + (a.q_valid ? min(max(a.q_valid[b], 0), a.Q) : a.Q) : n_q;
  const KVView& kv = a.kv;
  const int pt = paged ? kv.page_tokens : 1;
  const bf16_t* kslab = (const bf16_t*)kv.k;
  const bf16_t* vslab = (const bf16_t*)kv.v;
  const int32_t* table = paged ? kv.table + (int64_t)b * kv.max_pages : nullptr;
  // packed scratch: K [Hkv][tpad][DH], V [Hkv][DH][tpad], the sequence starts at column cu_pad[b]
  const int64_t pcol = paged ? 0 : kv.cu_pad[b];

  // query fragments: B operand, column c = row of this wave's tile
  u32x4 qf[QT][KK];
  int64_t row_out[QT];        // (token * Hq + head) of the lane's query, -1 if beyond R
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    int r = rg * 16 * QT + t * 16 + c;
    const bool ok = r < R;
    if (!ok) r = 0;
    const int hg = r / n_q, j = r - hg * n_q;
    const int64_t ro = (int64_t)(row_base + j) * a.Hq + kvh * G + hg;
    row_out[t] = ok ? ro : -1;
    const bf16_t* qp = a.q + ro * DH + g * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[t][kk] = *(const u32x4*)(qp + kk * 32);
  }

  f32x4 oacc[DT][QT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int t = 0; t < QT; ++t) oacc[d][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) { m_run[t] = -DEV_INF; l_run[t] = 0.f; }
  bool bad = false;

  // A wave takes its 32-key blocks two at a time: the page ids of both, then the K and V^T
  // fragments of both are requested before the first is multiplied, so the second block's two
  // memory round trips hide behind the first block's arithmetic (at batch 1 a wave owns about
  // two blocks and the kernel is a chain of latencies).
  struct Blk {
    u32x4 kf[2][KK];   // K fragments (A operand): tile tt row c <-> key k0 + 8*(c/4) + c%4 + 4*tt
    u32x4 vf[DT];      // V^T fragments (A operand of the second product): row = channel d*16 + c, keys k0+8g..+7
    bool pbad;         // the V page is not addressable
  };
  auto key_of = [&](int kb, int which) -> int {     // which: 0, 1 = K tiles, 2 = V; clamped into the sequence
    const int k0 = kb << 5;
    if (which < 2) {
      const int key = k0 + 8 * (c >> 2) + (c & 3) + 4 * which;
      return key < kv_len ? key : kv_len - 1;       // masked at the scores; keeps the load in bounds
    }
    const int key = k0 + 8 * g;
    return key < kv_len ? key : (kv_len - 1) & ~7;  // zeroed before use
  };
  auto pages = [&](int kb, int (&pg)[3]) {
    if (paged) {
#pragma unroll
      for (int x = 0; x < 3; ++x) {
        const int pi = key_of(kb, x) / pt;
        const int v = table[pi < kv.max_pages ? pi : kv.max_pages - 1];
        pg[x] = pi < kv.max_pages ? v : -1;
      }
    }
  };
  auto issue = [&](int kb, const int (&pg)[3], Blk& blk) {
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int key = key_of(kb, tt);
      const bf16_t* kp;
      if (paged) {
        const bool ok = (uint32_t)pg[tt] < (uint32_t)kv.n_pages;
        bad |= !ok;
        kp = kslab + (((int64_t)(ok ? pg[tt] : 0) * kv.n_kv_heads + kvh) * pt + (key - key / pt * pt)) * DH + g * 8;
      } else {
        kp = kslab + ((int64_t)kvh * kv.tpad + pcol + key) * DH + g * 8;
      }
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) blk.kf[tt][kk] = *(const u32x4*)(kp + kk * 32);
    }
    const int key = key_of(kb, 2);
    const bf16_t* vp;
    int64_t vstep;                                           // elements between channels d*16 and (d+1)*16
    blk.pbad = false;
    if (paged) {
      const bool ok = (uint32_t)pg[2] < (uint32_t)kv.n_pages;
      bad |= !ok;
      blk.pbad = !ok;
      vp = vslab + (((int64_t)(ok ? pg[2] : 0) * kv.n_kv_heads + kvh) * DH + c) * pt + (key - key / pt * pt);
      vstep = (int64_t)16 * pt;
    } else {
      vp = vslab + ((int64_t)kvh * DH + c) * kv.tpad + pcol + key;
      vstep = (int64_t)16 * kv.tpad;
    }
#pragma unroll
    for (int d = 0; d < DT; ++d) blk.vf[d] = *(const u32x4*)(vp + d * vstep);
  };
  auto compute = [&](int kb, Blk& blk) {
    const int k0 = kb << 5;
    if (__builtin_amdgcn_ballot_w64(blk.pbad) != 0 || k0 + 32 > kv_len) {
      // zero what lies beyond the sequence (or in a page that is not addressable): the slots may
      // hold anything, and 0 * NaN would poison the row
#pragma unroll
      for (int d = 0; d < DT; ++d) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uint32_t v = blk.vf[d][e];
          const int ke = k0 + 8 * g + 2 * e;
          if (blk.pbad || ke >= kv_len) v &= 0xffff0000u;
          if (blk.pbad || ke + 1 >= kv_len) v &= 0x0000ffffu;
          blk.vf[d][e] = v;
        }
      }
    }
    // ---- S^T tiles
    f32x4 s[2][QT];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) acc = mfma16(blk.kf[tt][kk], qf[t][kk], acc);
        s[tt][t] = acc;
      }
    // ---- online softmax per query column
    u32x4 pf[QT], pl[QT];
    attn_softmax_block<DT, QT>(s, k0, kv_len, g, a.scale_log2, m_run, l_run, oacc, pf, pl);
    // ---- O^T += V^T P^T
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        oacc[d][t] = mfma16(blk.vf[d], pf[t], oacc[d][t]);
        oacc[d][t] = mfma16(blk.vf[d], pl[t], oacc[d][t]);
      }
  };

  const int nkb = (kv_len + 31) >> 5;
  for (int kb = unit; kb < nkb; kb += 2 * a.n_units) {
    const int kb2 = kb + a.n_units;
    const bool two = kb2 < nkb;
    const int kbb = two ? kb2 : kb;               // a repeat of the first block's loads: no branch around a load
    int pga[3], pgb[3];
    pages(kb, pga);
    pages(kbb, pgb);
    Blk ba, bb;
    issue(kb, pga, ba);
    issue(kbb, pgb, bb);
    compute(kb, ba);
    if (two) compute(kb2, bb);
  }

  // ---- results: lane holds query column c, channels d*16 + 4g + i
  float l_red[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    l_red[t] = l;
  }
  auto store_out = [&](int d, int t, f32x4 v, float l) {       // normalised output, the row's only partial
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    const int64_t ro = row_out[t];
    const int tok = (int)(ro / a.Hq), head = (int)(ro - (int64_t)tok * a.Hq);
    const int ch = d * 16 + 4 * g;
    const int64_t at = a.out_mt > 0 ? frag_offset(tok, head * DH + ch, a.out_mt) : ro * DH + ch;
    *(uint2*)(a.o + at) = make_uint2(pack_bf16x2(v[0] * inv, v[1] * inv), pack_bf16x2(v[2] * inv, v[3] * inv));
  };
  if (a.kspl > 1) {
    // The workgroup's waves hold partial results of the same rows over different keys (launched only
    // with one row group per workgroup, so every wave is here): bring them to a common maximum,
    // park them in LDS and let each wave add up a slice of the channels, in wave order.
    const int KS = a.kspl;
    float* sm_m = (float*)attn_smem;                           // [KS][QT][16]
    float* sm_l = sm_m + KS * QT * 16;                         // [KS][QT][16]
    f32x4* sm_o = (f32x4*)(attn_smem + 2 * KS * QT * 16 * sizeof(float));   // [KS][DT*QT][64]
    if (g == 0) {
#pragma unroll
      for (int t = 0; t < QT; ++t) { sm_m[(w * QT + t) * 16 + c] = m_run[t]; sm_l[(w * QT + t) * 16 + c] = l_red[t]; }
    }
    __syncthreads();
    float m_all[QT], l_all[QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      float mx = -DEV_INF;
      for (int ww = 0; ww < KS; ++ww) mx = fmaxf(mx, sm_m[(ww * QT + t) * 16 + c]);
      float ls = 0.f;
      for (int ww = 0; ww < KS; ++ww) {
        const float mw = sm_m[(ww * QT + t) * 16 + c];
        ls += mw > -DEV_INF ? sm_l[(ww * QT + t) * 16 + c] * exp2f(mw - mx) : 0.f;
      }
      m_all[t] = mx;
      l_all[t] = ls;
      const float f = m_run[t] > -DEV_INF ? exp2f(m_run[t] - mx) : 0.f;
#pragma unroll
      for (int d = 0; d < DT; ++d) sm_o[(w * DT * QT + d * QT + t) * 64 + lane] = oacc[d][t] * f;
    }
    __syncthreads();
    for (int u = w; u < DT * QT; u += KS) {
      const int d = u / QT, t = u - d * QT;
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int ww = 0; ww < KS; ++ww) acc = acc + sm_o[(ww * DT * QT + u) * 64 + lane];
      if (row_out[t] < 0) continue;
      if (a.n_parts == 1) { store_out(d, t, acc, l_all[t]); continue; }
      const int64_t slot = row_out[t] * a.n_parts + blockIdx.x;
      *(f32x4*)(a.part_o + slot * DH + d * 16 + 4 * g) = acc;
      if (d == 0 && g == 0) { a.part_ml[slot * 2] = m_all[t]; a.part_ml[slot * 2 + 1] = l_all[t]; }
    }
  } else {
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      if (row_out[t] < 0) continue;
      if (a.n_parts == 1) {
#pragma unroll
        for (int d = 0; d < DT; ++d) store_out(d, t, oacc[d][t], l_red[t]);
        continue;
      }
      const int64_t slot = row_out[t] * a.n_parts + unit;
      float* po = a.part_o + slot * DH + 4 * g;
#pragma unroll
      for (int d = 0; d < DT; ++d) *(f32x4*)(po + d * 16) = oacc[d][t];
      if (g == 0) { a.part_ml[slot * 2] = m_run[t]; a.part_ml[slot * 2 + 1] = l_red[t]; }
    }
  }
  if (bad) atomicOr(a.status, DLLM_STATUS_BAD_PAGE);
}

// merges the units' partials of one (token, head) row and stores the normalised output
// (fragment order of the [T, Hq*DH] matrix: it is the activation operand of the output projection)
template <int DH>
__global__ __launch_bounds__(512) void k_attn_combine(const float* part_o, const float* part_ml, int n_units,
                                                      bf16_t* o, int Hq, int mt, int64_t n_rows) {
  const int64_t row = (int64_t)blockIdx.x * (512 / DH) + threadIdx.x / DH;
  if (row >= n_rows) return;
  const int d = threadIdx.x % DH;
  // eight units at a time: their loads are independent and issued together, the running
  // (max, numerator, denominator) is rescaled between chunks
  float M = -DEV_INF, num = 0.f, den = 0.f;
  for (int u0 = 0; u0 < n_units; u0 += 8) {
    float mu[8], lu[8], ou[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool ok = u0 + i < n_units;
      const int64_t slot = row * n_units + (ok ? u0 + i : n_units - 1);
      const float2 ml = *(const float2*)(part_ml + slot * 2);
      mu[i] = ok ? ml.x : -DEV_INF;
      lu[i] = ml.y;
      ou[i] = part_o[slot * DH + d];
    }
    float Mn = M;
#pragma unroll
    for (int i = 0; i < 8; ++i) Mn = fmaxf(Mn, mu[i]);
    if (Mn == -DEV_INF) continue;                       // nothing but empty units so far
    const float r = exp2f(M - Mn);                      // exp2(-inf) = 0 on the first chunk
    num *= r;
    den *= r;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float sc = exp2f(mu[i] - Mn);               // 0 for empty units
      den = fmaf(lu[i], sc, den);
      num = fmaf(ou[i], sc, num);
    }
    M = Mn;
  }
  const int tok = (int)(row / Hq), head = (int)(row - (int64_t)tok * Hq);
  const int64_t at = mt > 0 ? frag_offset(tok, head * DH + d, mt) : row * DH + d;
  o[at] = f32_to_bf16(den > 0.f ? num / den : 0.f);
}

// ------------------------------------------------------------------------------------------
// The same attention for many query rows per KV head (grouped-query models at large batch, and
// every no-cache forward): the waves of a workgroup are row groups of 32 rows that all need the
// same keys, so each 64-key block of K and V^T is fetched from memory once per workgroup, by all
// threads together, and laid out in LDS in operand order (every fragment read is 64 lanes x 16
// bytes of one KiB; inside the KiB the row index is xor-ed with the piece's column so that the
// loader's consecutive lanes, which walk along a row, hit different banks); two LDS buffers, the
// next block in flight in registers while the current one is multiplied.  Arithmetic, masking and
// outputs are those of k_attn_step.
template <int DH, int NW, bool PAGED, bool FAST>
__global__ __launch_bounds__(NW * 64) void k_attn_lds(const AttnArgs a) {
  constexpr int KK = DH / 32, DT = DH / 16, QT = 2;
  constexpr int KP = DH / 8;                 // 16-byte pieces of a K row
  constexpr int KPB = 64 * KP, VPB = DH * 8; // pieces of a 64-key block: K rows, V^T channel rows
  constexpr int NP = KPB + VPB, nthr = NW * 64, MAXP = NP / nthr;
  static_assert(KPB % nthr == 0 && VPB % nthr == 0, "a thread's i-th piece is K for all threads or V for all");
  __shared__ u32x4 sk[2][2][2][KK][64];      // [buffer][32-key half][tile][k-step][lane]
  __shared__ u32x4 sv[2][2][DT][64];         // [buffer][32-key half][channel tile][lane]
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int rg = blockIdx.y * a.n_rg_wg + w;
  const int unit = blockIdx.x;
  const int b = blockIdx.z / a.Hkv, kvh = blockIdx.z - b * a.Hkv;
  const int G = a.Hq / a.Hkv;
  const int row_base = PAGED ? b * a.Q : a.cu[b];
  const int n_q = PAGED ? a.Q : a.cu[b + 1] - a.cu[b];
  const int R = n_q * G;
  const int kv_len = PAGED ? a.prefix_len[b] + (a.q_valid ? min(max(a.q_valid[b], 0), a.Q) : a.Q) : n_q;
  const bool active = w < a.n_rg_wg && rg * 16 * QT < R;     // waves beyond the rows only help loading
  if (blockIdx.y * a.n_rg_wg * 16 * QT >= R) return;         // whole workgroup beyond this sequence's rows
  const KVView& kv = a.kv;
  const int sh = a.pt_shift, pt = 1 << sh;                   // page size (a power of two)
  const bf16_t* kslab = (const bf16_t*)kv.k;
  const bf16_t* vslab = (const bf16_t*)kv.v;
  const int32_t* table = PAGED ? kv.table + (int64_t)b * kv.max_pages : nullptr;
  const int64_t pcol = PAGED ? 0 : kv.cu_pad[b];
  bool bad = false;

  u32x4 qf[QT][KK];
  int64_t row_out[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    int r = rg * 16 * QT + t * 16 + c;
    const bool ok = active && r < R;
    if (!ok) r = 0;
    const int hg = r / n_q, j = r - hg * n_q;
    const int64_t ro = (int64_t)(row_base + j) * a.Hq + kvh * G + hg;
    row_out[t] = ok ? ro : -1;
    const bf16_t* qp = a.q + ro * DH + g * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[t][kk] = *(const u32x4*)(qp + kk * 32);
  }

  // ---- cooperative loader.  Piece p = tid + i * nthr of a 64-key block: a 16-byte column of a K
  // row (i-th pieces below KPB) or eight keys of a V^T channel row.  No branch anywhere on the
  // way to a load, and the page ids of a block are fetched one block earlier than its data, so a
  // wave never waits on two dependent memory round trips.
  auto piece_key = [&](int i, int kb64) -> int {              // first key the piece addresses (clamped into the sequence)
    const int p = tid + i * nthr;
    if (i * nthr < KPB) {
      const int key = (kb64 << 6) + p / KP;
      return key < kv_len ? key : kv_len - 1;                   // masked at the scores
    }
    const int key = (kb64 << 6) + ((p - KPB) & 7) * 8;
    return key < kv_len ? key : (kv_len - 1) & ~7;              // zeroed when it is put into LDS
  };
  // FAST: a 64-key block lies inside one page (page size a multiple of 64) or in the packed scratch, so
  // its K rows are 64 * DH contiguous elements and its V^T rows 64 contiguous keys per channel: one
  // base per block (wave-uniform) plus a per-thread constant.  Rows past the sequence end are read
  // as they are (inside the page, or inside the workspace) and masked or zeroed later.
  int koff[MAXP];
#pragma unroll
  for (int i = 0; i < MAXP; ++i) {
    const int p = tid + i * nthr;
    if (i * nthr < KPB) koff[i] = p * 8;
    else koff[i] = ((p - KPB) >> 3) * (PAGED ? pt : kv.tpad) + ((p - KPB) & 7) * 8;
  }
  auto fetch_pages = [&](int (&pg)[MAXP], int kb64) {
    if constexpr (PAGED && FAST) {
      const int pi = (kb64 << 6) >> sh;
      const int v = table[pi < kv.max_pages ? pi : kv.max_pages - 1];
      pg[0] = pi < kv.max_pages ? v : -1;
    } else if constexpr (PAGED) {
#pragma unroll
      for (int i = 0; i < MAXP; ++i) {
        const int pi = piece_key(i, kb64) >> sh;
        const int v = table[pi < kv.max_pages ? pi : kv.max_pages - 1];
        pg[i] = pi < kv.max_pages ? v : -1;
      }
    }
  };
  auto issue = [&](u32x4 (&reg)[MAXP], const int (&pg)[MAXP], int kb64, uint32_t& vbad) {
    vbad = 0;
    if constexpr (FAST) {
      const int k0 = kb64 << 6;
      int64_t kb, vb;
      if constexpr (PAGED) {
        const int page = __builtin_amdgcn_readfirstlane(pg[0]);
        const bool ok = (uint32_t)page < (uint32_t)kv.n_pages;
        bad |= !ok;
        vbad = ok ? 0u : 0xffffffffu;
        const int64_t rows = (((int64_t)(ok ? page : 0) * kv.n_kv_heads + kvh) << sh);
        kb = (rows + (k0 & (pt - 1))) * DH;
        vb = rows * DH + (k0 & (pt - 1));
      } else {
        kb = ((int64_t)kvh * kv.tpad + pcol + k0) * DH;
        vb = (int64_t)kvh * DH * kv.tpad + pcol + k0;
      }
      const bf16_t* kp = kslab + kb;
      const bf16_t* vp = vslab + vb;
#pragma unroll
      for (int i = 0; i < MAXP; ++i) reg[i] = *(const u32x4*)((i * nthr < KPB ? kp : vp) + koff[i]);
      return;
    }
#pragma unroll
    for (int i = 0; i < MAXP; ++i) {
      const int p = tid + i * nthr;
      const int key = piece_key(i, kb64);
      int64_t off;
      if (i * nthr < KPB) {
        const int pc = p % KP;
        if constexpr (PAGED) {
          const bool ok = (uint32_t)pg[i] < (uint32_t)kv.n_pages;
          bad |= !ok;
          off = ((((int64_t)(ok ? pg[i] : 0) * kv.n_kv_heads + kvh) << sh) + (key & (pt - 1))) * DH + pc * 8;
        } else {
          off = ((int64_t)kvh * kv.tpad + pcol + key) * DH + pc * 8;
        }
        reg[i] = *(const u32x4*)(kslab + off);
      } else {
        const int ch = (p - KPB) >> 3;
        if constexpr (PAGED) {
          const bool ok = (uint32_t)pg[i] < (uint32_t)kv.n_pages;
          bad |= !ok;
          vbad |= ok ? 0u : (1u << i);
          off = ((((int64_t)(ok ? pg[i] : 0) * kv.n_kv_heads + kvh) * DH + ch) << sh) + (key & (pt - 1));
        } else {
          off = ((int64_t)kvh * DH + ch) * kv.tpad + pcol + key;
        }
        reg[i] = *(const u32x4*)(vslab + off);
      }
    }
  };
  // V^T elements of keys beyond the sequence (or of a page that is not addressable) become zero
  // here: their probability is zero, and zero times whatever the pool holds there must stay zero
  auto commit = [&](const u32x4 (&reg)[MAXP], int buf, int kb64, uint32_t vbad) {
    u32x4* dk = &sk[buf][0][0][0][0];
    u32x4* dv = &sv[buf][0][0][0];
    const bool fix = (kb64 << 6) + 64 > kv_len || __builtin_amdgcn_ballot_w64(vbad != 0) != 0;
#pragma unroll
    for (int i = 0; i < MAXP; ++i) {
      const int p = tid + i * nthr;
      if (i * nthr < KPB) {
        const int r = p / KP, pc = p - r * KP;
        const int half = r >> 5, r32 = r & 31, aa = r32 >> 3, bb = r32 & 7;
        const int tt = bb >> 2, cc = 4 * aa + (bb & 3);         // key 8a+b of a half sits in tile b/4, row 4a + b%4
        dk[(((half * 2 + tt) * KK + (pc >> 2)) * 64) + (pc & 3) * 16 + (cc ^ (4 * (pc & 3)) ^ (pc >> 2))] = reg[i];
      } else {
        const int q = p - KPB, ch = q >> 3, kg = q & 7;
        u32x4 v = reg[i];
        if (fix) {                                              // only a sequence's last block, or a bad page
          int valid = kv_len - ((kb64 << 6) + kg * 8);          // elements of this piece inside the sequence
          if (vbad & (1u << i)) valid = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            uint32_t x = v[e];
            x = valid > 2 * e + 1 ? x : (x & 0x0000ffffu);
            x = valid > 2 * e ? x : 0u;
            v[e] = x;
          }
        }
        dv[(((kg >> 2) * DT + (ch >> 4)) * 64) + (kg & 3) * 16 + ((ch & 15) ^ (4 * (kg & 3)) ^ (2 * (kg >> 2)))] = v;
      }
    }
  };

  f32x4 oacc[DT][QT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int t = 0; t < QT; ++t) oacc[d][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) { m_run[t] = -DEV_INF; l_run[t] = 0.f; }

  auto compute = [&](int buf, int kb64) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int k0 = (kb64 << 6) + half * 32;
      if (k0 >= kv_len) break;
      f32x4 s[2][QT];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        u32x4 kf[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[kk] = sk[buf][half][tt][kk][lane ^ (4 * g) ^ kk];
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) acc = mfma16(kf[kk], qf[t][kk], acc);
          s[tt][t] = acc;
        }
      }
      u32x4 pf[QT], pl[QT];
      attn_softmax_block<DT, QT>(s, k0, kv_len, g, a.scale_log2, m_run, l_run, oacc, pf, pl);
#pragma unroll
      for (int d = 0; d < DT; ++d) {
        const u32x4 vf = sv[buf][half][d][lane ^ (4 * g) ^ (2 * half)];
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          oacc[d][t] = mfma16(vf, pf[t], oacc[d][t]);
          oacc[d][t] = mfma16(vf, pl[t], oacc[d][t]);
        }
      }
    }
  };

  const int nkb = (kv_len + 63) >> 6;
  if (unit < nkb) {
    const int last = unit + ((nkb - 1 - unit) / a.n_units) * a.n_units;
    u32x4 reg[MAXP];
    int pg[MAXP];
    uint32_t vbad;
    fetch_pages(pg, unit);
    issue(reg, pg, unit, vbad);
    {
      const int nxt = unit + a.n_units;
      fetch_pages(pg, nxt <= last ? nxt : last);
    }
    commit(reg, 0, unit, vbad);
    int buf = 0;
    for (int kb = unit; kb < nkb; kb += a.n_units) {
      __syncthreads();
      int nxt = kb + a.n_units;
      nxt = nxt <= last ? nxt : last;
      int nxt2 = nxt + a.n_units;
      nxt2 = nxt2 <= last ? nxt2 : last;
      issue(reg, pg, nxt, vbad);          // its page ids arrived during the previous block
      fetch_pages(pg, nxt2);
      if (active) compute(buf, kb);
      commit(reg, buf ^ 1, nxt, vbad);
      buf ^= 1;
    }
  }

  if (active) {
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      float l = l_run[t];
      l += __shfl_xor(l, 16, 64);
      l += __shfl_xor(l, 32, 64);
      if (row_out[t] < 0) continue;
      if (a.n_units == 1) {
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        const int64_t ro = row_out[t];
        const int tok = (int)(ro / a.Hq), head = (int)(ro - (int64_t)tok * a.Hq);
#pragma unroll
        for (int d = 0; d < DT; ++d) {
          const int ch = d * 16 + 4 * g;
          const int64_t at = a.out_mt > 0 ? frag_offset(tok, head * DH + ch, a.out_mt) : ro * DH + ch;
          *(uint2*)(a.o + at) = make_uint2(
              (uint32_t)f32_to_bf16(oacc[d][t][0] * inv) | ((uint32_t)f32_to_bf16(oacc[d][t][1] * inv) << 16),
              (uint32_t)f32_to_bf16(oacc[d][t][2] * inv) | ((uint32_t)f32_to_bf16(oacc[d][t][3] * inv) << 16));
        }
        continue;
      }
      const int64_t slot = row_out[t] * a.n_units + unit;
      float* po = a.part_o + slot * DH + 4 * g;
#pragma unroll
      for (int d = 0; d < DT; ++d) *(f32x4*)(po + d * 16) = oacc[d][t];
      if (g == 0) { a.part_ml[slot * 2] = m_run[t]; a.part_ml[slot * 2 + 1] = l; }
    }
  }
  if (bad) atomicOr(a.status, DLLM_STATUS_BAD_PAGE);
}

bool attn_step_supported(const dllm_ctx* c, const StepGeom& g) {
  const dllm_config& f = c->cfg;
  if (!(f.dtype == DLLM_BF16 && c->kernel_mode == 0 && c->map.attn_rows > 0)) return false;
  return g.Q > 0 ? f.page_tokens % 8 == 0 : true;
}

// Attention of a denoise step (paged pool) or of a no-cache forward (packed scratch).
// merging four waves' partial results takes a little more LDS than a kernel gets by default
static bool attn_merge_ready = false;
hipError_t init_attn_kernels() {
  if (attn_merge_ready) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)k_attn_step<128, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_attn_step<64, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
  attn_merge_ready = e == hipSuccess;
  return e;
}

hipError_t launch_attn_step(dllm_ctx* c, hipStream_t s, const StepGeom& g, const KVView& kv, bool frag_out) {
  const dllm_config& f = c->cfg;
  const int G = f.n_q_heads / f.n_kv_heads;
  const int max_q = g.Q > 0 ? g.Q : g.max_kv;                 // most query rows of a sequence
  const int R = max_q * G;
  constexpr int QT = 2;
  const int n_rg = (R + 16 * QT - 1) / (16 * QT);
  static const int no_lds = getenv("DLLM_NO_ATTN_LDS") ? 1 : 0;   // tuning aid
  int pt_shift = 0;
  if (g.Q > 0) {
    pt_shift = -1;
    for (int sft = 3; sft < 31; ++sft) if (f.page_tokens == (1 << sft)) pt_shift = sft;
  }
  const bool staged = n_rg >= 4 && !no_lds && pt_shift >= 0;   // K/V staged in LDS, up to 8 row groups per workgroup
  const int rg_cap = staged ? 8 : 4;                           // the register-direct kernel runs at most 4 waves
  const int n_rg_wg = n_rg < rg_cap ? n_rg : rg_cap;
  const int n_chunks = (n_rg + n_rg_wg - 1) / n_rg_wg;
  const int nkb = (g.max_kv + 31) / 32;
  // units along the keys: short dependent chains matter more than partial traffic here (a step's
  // attention is a few MB), so give every unit about two 32-key blocks, within the partial buffer
  int64_t want = 2048 / ((int64_t)g.B * f.n_kv_heads * n_rg);
  if (want < 1) want = 1;
  int64_t by_work = staged ? (nkb + 7) / 8 : (nkb + 1) / 2;   // staged kernel: at least four 64-key blocks per unit
  int64_t by_space = c->map.attn_rows / ((int64_t)g.T * f.n_q_heads);
  int64_t units = want < by_work ? want : by_work;
  if (units > by_space) units = by_space;
  if (units > ATTN_MAX_SPLITS) units = ATTN_MAX_SPLITS;
  if (units < 1) units = 1;                                   // a single unit needs no partial buffer
  // one row group per KV head (a batch-1 block on a multi-head model): four units share a workgroup and
  // merge their partial results in LDS, which leaves a quarter of the partials to write and re-read
  int kspl = 1;
  if (!staged && n_rg == 1 && attn_merge_ready && units >= 4) {
    kspl = 4;
    int64_t parts = (nkb + 2 * kspl - 1) / (2 * kspl);
    if (parts * kspl > want) parts = want / kspl;
    if (parts > by_space) parts = by_space;
    if (parts < 1) parts = 1;
    units = parts * kspl;
  }
  AttnArgs a;
  a.q = WSM(c, q, bf16_t);
  a.prefix_len = g.prefix_len;
  a.q_valid = g.Q > 0 ? g.q_valid : nullptr;
  a.cu = g.cu_seqlens;
  a.o = WSM(c, o, bf16_t);
  a.out_mt = frag_out ? (g.T + 15) / 16 : 0;
  a.kv = kv;
  a.Q = g.Q; a.Hq = f.n_q_heads; a.Hkv = f.n_kv_heads; a.B = g.B;
  a.n_units = (int)units; a.kspl = kspl; a.n_rg_wg = n_rg_wg;
  a.n_parts = (int)(units / kspl);
  a.pt_shift = pt_shift;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)f.head_dim);
  a.part_o = WSM(c, attn_part, float);
  a.part_ml = a.part_o + (size_t)c->map.attn_rows * f.head_dim;
  a.status = WSM(c, status, int32_t);
  dim3 grid((unsigned)(units / kspl), n_chunks, g.B * f.n_kv_heads);
  const int threads = 64 * n_rg_wg * kspl;
  if (staged) {
    // many rows per kv head: K/V staged once per workgroup in LDS (at least 4 waves load)
    const bool paged = g.Q > 0;
    const bool fast = !paged || a.pt_shift >= 6;     // a 64-key block never straddles pages
#define ATTN_LDS(DHV, NWV)                                                                                 \
  do {                                                                                                     \
    if (!paged) k_attn_lds<DHV, NWV, false, true><<<grid, NWV * 64, 0, s>>>(a);                            \
    else if (fast) k_attn_lds<DHV, NWV, true, true><<<grid, NWV * 64, 0, s>>>(a);                          \
    else k_attn_lds<DHV, NWV, true, false><<<grid, NWV * 64, 0, s>>>(a);                                   \
  } while (0)
    if (f.head_dim == 128) {
      if (n_rg_wg <= 4) ATTN_LDS(128, 4); else ATTN_LDS(128, 8);
    } else {
      if (n_rg_wg <= 4) ATTN_LDS(64, 4); else ATTN_LDS(64, 8);
    }
#undef ATTN_LDS
  } else {
    const size_t lds = kspl > 1 ? (size_t)kspl * (2 * QT * 16 * sizeof(float) + (size_t)(f.head_dim / 16) * QT * 64 * 16) : 0;
    if (f.head_dim == 128) k_attn_step<128, QT><<<grid, threads, lds, s>>>(a);
    else k_attn_step<64, QT><<<grid, threads, lds, s>>>(a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.n_parts == 1) return e;
  const int rows = g.T * f.n_q_heads;
  if (f.head_dim == 128)
    k_attn_combine<128><<<(rows + 3) / 4, 512, 0, s>>>(a.part_o, a.part_ml, a.n_parts, a.o, f.n_q_heads, a.out_mt, rows);
  else
    k_attn_combine<64><<<(rows + 7) / 8, 512, 0, s>>>(a.part_o, a.part_ml, a.n_parts, a.o, f.n_q_heads, a.out_mt, rows);
  return hipGetLastError();
}

}  // namespace dllm

// ==========================================================================================
// Large-M bfloat16 GEMM on the matrix cores: C[M,N] = A[M,K] * W[N,K]^T (both K-contiguous).
// A workgroup of 4 waves computes a BM x 128 tile (BM = 256 or 128 token rows; waves 2x2, each
// BM/2 x 64), 64-deep K slices are staged through LDS in fragment order (every operand read is 64
// lanes x 16 contiguous bytes, no bank conflicts), double-buffered in LDS and double-buffered in
// registers on the way there, so two slices are in flight from memory while a third is multiplied.
// The weight tile is the A operand of the instruction: a lane ends up with 4 consecutive output
// features of one token row (vector stores).  Epilogues: store, residual add, SiLU(gate)*up over two
// weight matrices, and the softmax statistics of the LM head per 64 columns.
namespace dllm {

constexpr int LG_BN = 128, LG_BK = 64;
// Inside a fragment's KiB in LDS the unit of (k-group g, row c) of k-step ks sits at g*16 + (c ^ lg_swz(g, ks)):
// reads stay a permutation of the KiB, and the loader's 16 consecutive lanes (two rows x eight
// 16-byte columns of a slice) write 16 different bank groups instead of two.
__device__ __forceinline__ int lg_swz(int g, int ks) { return (4 * g) ^ (2 * ks); }
enum LgEpi { LG_STORE = 0, LG_STORE_F32 = 1, LG_RESID = 2, LG_SWIGLU = 3, LG_LMSTATS = 4, LG_QKV = 5 };

struct LgArgs {
  const bf16_t* A;
  const bf16_t* W;
  const bf16_t* W2;        // SWIGLU: up projection; QKV: key projection
  const bf16_t* W3;        // QKV: value projection
  void* C;
  void* C2;                // QKV: float keys
  void* C3;                // QKV: bfloat16 values
  int N2, tiles_n1, tiles_n2;   // QKV: width of the key/value projections, column tiles of q and of k
  int k_per;               // RESID: K range of one split (multiple of LG_BK); gridDim.y splits
  int k_splits;            // 256-row kernel: number of K splits (its grid is flat)
  float* delta;            // RESID: products of splits 1.. go to delta[(split - 1) * delta_stride + m * N + n]
  int64_t delta_stride;
  const int32_t* m_dev;    // optional device row count
  int M, N, K, tiles_m, tiles_n;
  float* part;             // LMSTATS: [rows, n_parts, 4]
  int n_parts;
  int32_t mask_id;
};

template <int BM, int EPI>
__global__ __launch_bounds__(256) void k_gemm_mfma(const LgArgs a) {
  constexpr int TM = BM / 16;                 // 16-row token tiles of the block
  constexpr int WT = BM / 32;                 // token tiles per wave
  constexpr int NW2 = 1;
  constexpr int TILE_N = (EPI == LG_SWIGLU) ? LG_BN / 2 : LG_BN;   // output features of a tile
  constexpr int PA = BM / 32;                 // 16-byte pieces of A per thread and slice (BM*8/256)
  __shared__ u32x4 sa[2][2][TM][64];          // [buffer][k-step][token tile][lane]
  __shared__ u32x4 sw[2][NW2][2][8][64];      // [buffer][matrix][k-step][weight tile][lane]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  int M = a.M;
  if (a.m_dev) { const int md = *a.m_dev; M = md < M ? md : M; }
  int N = a.N;
  const int K = a.K;
  // XCD-aware tile order: workgroups are dealt round-robin to the 8 XCDs, so give each XCD a
  // contiguous run of tiles (m fastest) and let its L2 keep the weight block they share
  const int n_tiles = a.tiles_m * a.tiles_n;
  const int per_xcd = (n_tiles + 7) / 8;
  const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile >= n_tiles) return;
  int tn = tile / a.tiles_m;
  const int tm = tile - tn * a.tiles_m;
  // QKV: the column tiles of the three projections follow each other; a tile belongs to one of them
  const bf16_t* Wsel = a.W;
  void* Csel = a.C;
  bool out_f32 = EPI == LG_STORE_F32;
  if constexpr (EPI == LG_QKV) {
    out_f32 = true;
    if (tn >= a.tiles_n1 + a.tiles_n2) { tn -= a.tiles_n1 + a.tiles_n2; Wsel = a.W3; Csel = a.C3; N = a.N2; out_f32 = false; }
    else if (tn >= a.tiles_n1) { tn -= a.tiles_n1; Wsel = a.W2; Csel = a.C2; N = a.N2; }
  }
  const int m0 = tm * BM, n0 = tn * TILE_N;
  if (m0 >= M) return;
  // RESID: this workgroup's share of K
  int k_begin = 0, k_end = K;
  if constexpr (EPI == LG_RESID) {
    k_begin = blockIdx.y * a.k_per;
    k_end = k_begin + a.k_per < K ? k_begin + a.k_per : K;
  }
  const int wm = (w & 1) * (BM / 2), wn = (w >> 1) * 64;

  // loader: piece p = tid + 256*q of a [rows][8 pieces] slice: row p/8, 16-byte column p%8
  const bf16_t* ga[PA];
  const bf16_t* gw[NW2][4];
  int dsta[PA], dstw[4], kca[PA], kcw[4];
#pragma unroll
  for (int q = 0; q < PA; ++q) {
    const int p = tid + 256 * q, r = p >> 3, kc = p & 7;
    kca[q] = kc * 8;
    dsta[q] = ((kc >> 2) * TM + (r >> 4)) * 64 + (kc & 3) * 16 + ((r & 15) ^ lg_swz(kc & 3, kc >> 2));
    int ra = m0 + r; ra = ra < M ? ra : M - 1;
    ga[q] = a.A + (int64_t)ra * K;
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int p = tid + 256 * q, r = p >> 3, kc = p & 7;
    kcw[q] = kc * 8;
    dstw[q] = ((kc >> 2) * 8 + (r >> 4)) * 64 + (kc & 3) * 16 + ((r & 15) ^ lg_swz(kc & 3, kc >> 2));
    if constexpr (EPI == LG_SWIGLU) {
      // a wave's four weight tiles are gate, gate, up, up of the same 32 features: both factors of
      // silu(gate) * up meet in one lane
      int rw = n0 + (r >> 6) * 32 + ((r >> 4) & 1) * 16 + (r & 15); rw = rw < N ? rw : N - 1;
      gw[0][q] = (((r >> 5) & 1) ? a.W2 : a.W) + (int64_t)rw * K;
    } else {
      int rw = n0 + r; rw = rw < N ? rw : N - 1;
      gw[0][q] = Wsel + (int64_t)rw * K;
    }
  }
  struct Stage { u32x4 ra[PA]; u32x4 rw[NW2][4]; };
  auto issue = [&](Stage& st, int k0) {   // loads are clamped, never branched
#pragma unroll
    for (int q = 0; q < PA; ++q) {
      int k = k0 + kca[q];
      const bool ok = k + 8 <= k_end;
      k = ok ? k : K - 8;
      const u32x4 v = *(const u32x4*)(ga[q] + k);
      st.ra[q] = ok ? v : u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int x = 0; x < NW2; ++x)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        int k = k0 + kcw[q];
        const bool ok = k + 8 <= k_end;
        k = ok ? k : K - 8;
        const u32x4 v = *(const u32x4*)(gw[x][q] + k);
        st.rw[x][q] = ok ? v : u32x4{0, 0, 0, 0};
      }
  };
  auto commit = [&](const Stage& st, int buf) {
    u32x4* da = &sa[buf][0][0][0];
#pragma unroll
    for (int q = 0; q < PA; ++q) da[dsta[q]] = st.ra[q];
#pragma unroll
    for (int x = 0; x < NW2; ++x) {
      u32x4* dw = &sw[buf][x][0][0][0];
#pragma unroll
      for (int q = 0; q < 4; ++q) dw[dstw[q]] = st.rw[x][q];
    }
  };

  f32x4 acc[NW2][4][WT];   // [matrix][weight 16-row tile][token 16-row tile]
#pragma unroll
  for (int x = 0; x < NW2; ++x)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < WT; ++j) acc[x][i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](int buf) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      u32x4 fa[WT];
#pragma unroll
      for (int j = 0; j < WT; ++j) fa[j] = sa[buf][ks][(wm >> 4) + j][lane ^ lg_swz(g, ks)];
#pragma unroll
      for (int x = 0; x < NW2; ++x) {
        u32x4 fw[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) fw[i] = sw[buf][x][ks][(wn >> 4) + i][lane ^ lg_swz(g, ks)];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < WT; ++j) acc[x][i][j] = mfma16(fw[i], fa[j], acc[x][i][j]);
      }
    }
  };

  const int nk = (k_end - k_begin + LG_BK - 1) / LG_BK;
  const int last = nk - 1;
  Stage s0, s1;
  issue(s0, k_begin);
  issue(s1, k_begin + (1 < last ? 1 : last) * LG_BK);
  commit(s0, 0);
  // slice kt is multiplied from LDS[kt&1] while slice kt+1 waits in registers and slice kt+2 is in flight
  for (int kt = 0; kt < nk; kt += 2) {
    __syncthreads();
    issue(s0, k_begin + (kt + 2 < last ? kt + 2 : last) * LG_BK);
    compute(0);
    commit(s1, 1);
    __syncthreads();
    issue(s1, k_begin + (kt + 3 < last ? kt + 3 : last) * LG_BK);
    if (kt + 1 < nk) compute(1);
    commit(s0, 0);
  }

  // lane holds token column c of token tile j, features 4g..4g+3 of weight tile i
  if (EPI == LG_SWIGLU) {
#pragma unroll
    for (int j = 0; j < WT; ++j) {
      const int m = m0 + wm + j * 16 + c;
      if (m >= M) continue;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int n = n0 + (wn >> 1) + i * 16 + 4 * g;
        f32x4 v = acc[0][i][j];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = v[e] / (1.0f + expf(-v[e])) * acc[0][i + 2][j][e];
        if (n + 4 <= N) {
          *(uint2*)((bf16_t*)a.C + (int64_t)m * N + n) =
              make_uint2((uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16),
                         (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16));
        } else {
          for (int e = 0; e < 4 && n + e < N; ++e) ((bf16_t*)a.C)[(int64_t)m * N + n + e] = f32_to_bf16(v[e]);
        }
      }
    }
    return;
  }
  if (EPI == LG_LMSTATS) {
#pragma unroll
    for (int j = 0; j < WT; ++j) {
      const int m = m0 + wm + j * 16 + c;
      RowStat st;
      st.init();
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int n = n0 + wn + i * 16 + 4 * g + e;
          if (n < N && n != a.mask_id) st.merge(acc[0][i][j][e], n, 1.0f, acc[0][i][j][e]);
        }
#pragma unroll
      for (int o = 16; o < 64; o <<= 1) {
        const float m2 = __shfl_xor(st.m, o, 64), s2 = __shfl_xor(st.s, o, 64), t2 = __shfl_xor(st.t, o, 64);
        const int i2 = __shfl_xor(st.idx, o, 64);
        st.merge(m2, i2, s2, t2);
      }
      if (g == 0 && m < M && n0 + wn < N) {
        float* o = a.part + ((int64_t)m * a.n_parts + (n0 + wn) / 64) * 4;
        *(f32x4*)o = f32x4{st.m, __int_as_float(st.idx), st.s, st.t};
      }
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < WT; ++j) {
    const int m = m0 + wm + j * 16 + c;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = n0 + wn + i * 16 + 4 * g;
      f32x4 v = acc[0][i][j];
      if (n + 4 <= N) {
        const int64_t at = (int64_t)m * N + n;
        if (EPI == LG_RESID) {
          if (blockIdx.y == 0) {
            f32x4* p = (f32x4*)((float*)a.C + at);
            *p = *p + v;
          } else {
            *(f32x4*)(a.delta + (int64_t)(blockIdx.y - 1) * a.delta_stride + at) = v;
          }
        } else if (out_f32) {
          *(f32x4*)((float*)Csel + at) = v;
        } else {
          *(uint2*)((bf16_t*)Csel + at) = make_uint2((uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16),
                                                     (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16));
        }
      } else {
        for (int e = 0; e < 4; ++e) {
          if (n + e >= N) break;
          const int64_t at = (int64_t)m * N + n + e;
          if (EPI == LG_RESID) {
            if (blockIdx.y == 0) ((float*)a.C)[at] += v[e];
            else a.delta[(int64_t)(blockIdx.y - 1) * a.delta_stride + at] = v[e];
          } else if (out_f32) ((float*)Csel)[at] = v[e];
          else ((bf16_t*)Csel)[at] = f32_to_bf16(v[e]);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// The same products for at least 256 token rows, arranged for one wave per SIMD: a workgroup of 4
// waves owns a 256 x 256 tile, each wave 128 x 128 of it as 4 x 4 instructions of 32 x 32 x 16 with
// the 256 accumulator registers in the accumulation file.  Both operands stay row-major in memory
// and are copied straight into LDS (no register pass) in 32-deep K stages of a 4-stage ring, 16 rows
// x 64 bytes per wave instruction, the 16-byte pieces of a row xor-ed with bits 2..3 of the row so
// that a fragment read (32 rows x one piece) touches every bank once.  Per stage a wave issues its
// share of the copies for three stages ahead and reads the next operands between the products of
// the current ones; the only wait on memory is "the stage after this one has landed", once per
// stage, in the middle of the products.
constexpr int T2_NS = 4, T2_STAGE = 32768, T2_LDS = T2_NS * T2_STAGE;
#define T2_VMCNT(n) (((n) & 15) | (((n) >> 4) << 14) | 0x0F70)
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void t2_copy16(const void* g, void* l) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}

template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_t256(const LgArgs a) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char t2_smem[];
  unsigned char* smem = t2_smem;
  constexpr int TILE_N = (EPI == LG_SWIGLU) ? 128 : 256;      // output features of a tile
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int M = a.M;
  if (a.m_dev) { const int md = *a.m_dev; M = md < M ? md : M; }
  const int N = a.N, K = a.K;
  const int wm = w & 1, wn = w >> 1;
  const int r = lane & 31, h = lane >> 5;
  // Persistent workgroups, one per CU: the work items (K split, column tile, row tile - row tile
  // fastest, only row tiles that hold rows) are dealt in contiguous runs to the 8 XCDs (workgroups
  // go round-robin to XCDs), inside an XCD round-robin to its workgroups, so the row tiles that
  // share a weight tile run at the same time next to the same L2.
  const int tiles_m = (M + 255) / 256;
  const int n_tiles = tiles_m * a.tiles_n;
  const int n_items = n_tiles * a.k_splits;
  const int per_xcd = (n_items + 7) / 8;
  for (int iw = blockIdx.x >> 3; iw < per_xcd; iw += gridDim.x >> 3) {
  const int item = (blockIdx.x & 7) * per_xcd + iw;
  if (item >= n_items) break;
  const int split = item / n_tiles, tile = item - split * n_tiles;
  const int tn = tile / tiles_m, tm = tile - tn * tiles_m;
  const int m0 = tm * 256, n0 = tn * TILE_N;
  int k_begin = 0, k_end = K;
  if constexpr (EPI == LG_RESID || EPI == LG_QKV) {
    k_begin = split * a.k_per;
    k_end = k_begin + a.k_per < K ? k_begin + a.k_per : K;
  }
  // the ring is free once every wave has read the previous item's last operands
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  // copies: instruction q of this wave covers rows (w*4 + q%4)*16 .. +15 of the token part (q < 4) or of
  // the weight part; lane p: row p/4, LDS piece p%4 holds source piece (p%4) ^ ((row>>2)&3)
  const bf16_t* gsrc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int r = (w * 4 + (q & 3)) * 16 + (lane >> 2);
    const int piece = (lane & 3) ^ ((r >> 2) & 3);
    if (q < 4) {
      int row = m0 + r; row = row < M ? row : M - 1;
      gsrc[q] = a.A + (int64_t)row * K + piece * 8;
    } else if constexpr (EPI == LG_SWIGLU) {
      // a wave's four weight tiles are gate, gate, up, up of the same 64 features
      int row = n0 + (r >> 7) * 64 + ((r >> 5) & 1) * 32 + (r & 31); row = row < N ? row : N - 1;
      gsrc[q] = (((r >> 6) & 1) ? a.W2 : a.W) + (int64_t)row * K + piece * 8;
    } else if constexpr (EPI == LG_QKV) {
      // three projections stacked along the features: q rows [0, N), then k and v with N2 rows each
      // (all multiples of 256, so a tile belongs to one of them)
      const int row = n0 + r;
      const bf16_t* wsel = row < N ? a.W : (row < N + a.N2 ? a.W2 : a.W3);
      const int lrow = row < N ? row : (row < N + a.N2 ? row - N : row - N - a.N2);
      gsrc[q] = wsel + (int64_t)lrow * K + piece * 8;
    } else {
      int row = n0 + r; row = row < N ? row : N - 1;
      gsrc[q] = a.W + (int64_t)row * K + piece * 8;
    }
  }
  // fragment reads: lane (r = l%32, h = l/32), k-step s of a stage: piece 2s + h
  int offA[2], offW[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int slotp = ((2 * ks + h) ^ ((r >> 2) & 3)) * 16;
    offA[ks] = (wm * 128 + r) * 64 + slotp;
    offW[ks] = 16384 + (wn * 128 + r) * 64 + slotp;
  }
  f32x16 acc[4][4];   // [weight tile][token tile]
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int ns = (k_end - k_begin) / 32;      // K ranges are multiples of 32 (checked on the host)
#define T2_MMA(ks, i, j)                                                                                          \
  acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[ks][i]),                    \
                                                      __builtin_bit_cast(bf16x8, fa[ks][j]), acc[i][j], 0, 0, 0)
  u32x4 fa[2][4], fw[2][4];
#pragma unroll
  for (int st = 0; st < T2_NS - 1; ++st) {
    const int kd = k_begin + (st < ns ? st : ns - 1) * 32;
#pragma unroll
    for (int q = 0; q < 8; ++q) t2_copy16(gsrc[q] + kd, smem + st * T2_STAGE + (q >> 2) * 16384 + (w * 4 + (q & 3)) * 1024);
  }
  __builtin_amdgcn_s_waitcnt(T2_VMCNT(8 * (T2_NS - 2)));
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    fa[0][j] = *(const u32x4*)(smem + offA[0] + j * 2048);
    fw[0][j] = *(const u32x4*)(smem + offW[0] + j * 2048);
  }
  for (int st = 0; st < ns; ++st) {
    const unsigned char* base = smem + (st % T2_NS) * T2_STAGE;
    const unsigned char* nbase = smem + ((st + 1) % T2_NS) * T2_STAGE;
    unsigned char* dbase = smem + ((st + T2_NS - 1) % T2_NS) * T2_STAGE;   // freed by the barrier of the stage before
    const int sn = st + T2_NS - 1;
    const int kd = k_begin + (sn < ns ? sn : ns - 1) * 32;                  // past the end: a repeat into a free slot
    // k-step 0: in the shadow of its products request the ring's next stage and read k-step 1's operands
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_barrier(0);
      T2_MMA(0, i, 0); T2_MMA(0, i, 1); T2_MMA(0, i, 2); T2_MMA(0, i, 3);
      t2_copy16(gsrc[2 * i] + kd, dbase + ((2 * i) >> 2) * 16384 + (w * 4 + ((2 * i) & 3)) * 1024);
      t2_copy16(gsrc[2 * i + 1] + kd, dbase + ((2 * i + 1) >> 2) * 16384 + (w * 4 + ((2 * i + 1) & 3)) * 1024);
      fa[1][i] = *(const u32x4*)(base + offA[1] + i * 2048);
      fw[1][i] = *(const u32x4*)(base + offW[1] + i * 2048);
      __builtin_amdgcn_sched_barrier(0);
    }
    // k-step 1: wait until every wave's copies of the next stage have landed (all but the two
    // youngest stages of this wave's own), then read that stage's first operands
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_barrier(0);
      T2_MMA(1, i, 0); T2_MMA(1, i, 1); T2_MMA(1, i, 2); T2_MMA(1, i, 3);
      if (i == 0) {
        __builtin_amdgcn_s_waitcnt(T2_VMCNT(8 * (T2_NS - 2)));
        __builtin_amdgcn_s_barrier();
      }
      if (i == 1) { fa[0][0] = *(const u32x4*)(nbase + offA[0]); fa[0][1] = *(const u32x4*)(nbase + offA[0] + 2048); fa[0][2] = *(const u32x4*)(nbase + offA[0] + 4096); }
      if (i == 2) { fa[0][3] = *(const u32x4*)(nbase + offA[0] + 6144); fw[0][0] = *(const u32x4*)(nbase + offW[0]); fw[0][1] = *(const u32x4*)(nbase + offW[0] + 2048); }
      if (i == 3) { fw[0][2] = *(const u32x4*)(nbase + offW[0] + 4096); fw[0][3] = *(const u32x4*)(nbase + offW[0] + 6144); }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#undef T2_MMA
  __builtin_amdgcn_s_waitcnt(T2_VMCNT(0));   // the ring's trailing repeats must not outlive the workgroup

  // lane holds token column l%32 of token tile j; features (e/4)*8 + (l/32)*4 + e%4 of weight tile i
  if constexpr (EPI == LG_LMSTATS) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + wm * 128 + j * 32 + r;
#pragma unroll
      for (int half = 0; half < 2; ++half) {      // 64 columns per partial
        // the lane's 32 logits of this partial: maximum first (columns ascend, so the first of equal
        // maxima is the lowest), then the two sums against it
        float mx = -DEV_INF;
        int ix = 0x7fffffff;
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int i = half * 2 + ii;
            const int n = n0 + wn * 128 + i * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
            const float z = acc[i][j][e];
            if (n < N && n != a.mask_id && z > mx) { mx = z; ix = n; }
          }
        RowStat st;
        st.init();
        if (ix != 0x7fffffff) {
          float se = 0.f, sz = 0.f;
#pragma unroll
          for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int i = half * 2 + ii;
              const int n = n0 + wn * 128 + i * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
              const float z = acc[i][j][e];
              const float ex = (n < N && n != a.mask_id) ? __builtin_amdgcn_exp2f((z - mx) * 1.4426950408889634f) : 0.f;
              se += ex;
              sz = fmaf(ex, z, sz);
            }
          st.m = mx; st.idx = ix; st.s = se; st.t = sz;
        }
        const float m2 = __shfl_xor(st.m, 32, 64), s2 = __shfl_xor(st.s, 32, 64), t2 = __shfl_xor(st.t, 32, 64);
        const int i2 = __shfl_xor(st.idx, 32, 64);
        st.merge(m2, i2, s2, t2);
        const int nb = n0 + wn * 128 + half * 64;
        if (h == 0 && m < M && nb < N) {
          float* o = a.part + ((int64_t)m * a.n_parts + nb / 64) * 4;
          *(f32x4*)o = f32x4{st.m, __int_as_float(st.idx), st.s, st.t};
        }
      }
    }
  } else {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int m = m0 + wm * 128 + j * 32 + r;
    if (m >= M) continue;
    if constexpr (EPI == LG_SWIGLU) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int n = n0 + wn * 64 + i * 32 + e4 * 8 + h * 4;
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float gt = acc[i][j][e4 * 4 + e];
            v[e] = gt * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gt)) * acc[i + 2][j][e4 * 4 + e];
          }
          if (n + 4 <= N) {
            *(uint2*)((bf16_t*)a.C + (int64_t)m * N + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
          } else {
            for (int e = 0; e < 4 && n + e < N; ++e) ((bf16_t*)a.C)[(int64_t)m * N + n + e] = f32_to_bf16(v[e]);
          }
        }
    } else if constexpr (EPI == LG_QKV) {
      // every split stores its partial sums: [split][row][q | k | v] floats
      const int nt = N + 2 * a.N2;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int n = n0 + wn * 128 + i * 32 + e4 * 8 + h * 4;
          *(f32x4*)(a.delta + (int64_t)split * a.delta_stride + (int64_t)m * nt + n) =
              f32x4{acc[i][j][e4 * 4], acc[i][j][e4 * 4 + 1], acc[i][j][e4 * 4 + 2], acc[i][j][e4 * 4 + 3]};
        }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int n = n0 + wn * 128 + i * 32 + e4 * 8 + h * 4;
          const f32x4 v = f32x4{acc[i][j][e4 * 4], acc[i][j][e4 * 4 + 1], acc[i][j][e4 * 4 + 2], acc[i][j][e4 * 4 + 3]};
          const int64_t at = (int64_t)m * N + n;
          if (n + 4 <= N) {
            if (split == 0) { f32x4* p = (f32x4*)((float*)a.C + at); *p = *p + v; }
            else *(f32x4*)(a.delta + (int64_t)(split - 1) * a.delta_stride + at) = v;
          } else {
            for (int e = 0; e < 4 && n + e < N; ++e) {
              if (split == 0) ((float*)a.C)[at + e] += v[e];
              else a.delta[(int64_t)(split - 1) * a.delta_stride + at + e] = v[e];
            }
          }
        }
    }
  }
  }   // store epilogues
  }   // work items
}

// the 256 x 256 form needs the whole ring in LDS: more than the default limit of a kernel
static bool t2_ready = false;
static int t2_cus = 256;
hipError_t init_gemm_t256() {
  if (t2_ready) return hipSuccess;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
        cus >= 8)
      t2_cus = cus / 8 * 8;
  }
  hipError_t e = hipFuncSetAttribute((const void*)k_gemm_t256<LG_RESID>, hipFuncAttributeMaxDynamicSharedMemorySize, T2_LDS);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_gemm_t256<LG_SWIGLU>, hipFuncAttributeMaxDynamicSharedMemorySize, T2_LDS);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_gemm_t256<LG_LMSTATS>, hipFuncAttributeMaxDynamicSharedMemorySize, T2_LDS);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_gemm_t256<LG_QKV>, hipFuncAttributeMaxDynamicSharedMemorySize, T2_LDS);
  t2_ready = e == hipSuccess;
  return e;
}

template <int EPI>
static hipError_t t2_launch(hipStream_t s, LgArgs a, int k_splits = 1) {
  constexpr int tile_n = EPI == LG_SWIGLU ? 128 : 256;
  a.tiles_m = (a.M + 255) / 256;
  a.tiles_n = (a.N + tile_n - 1) / tile_n;
  if (EPI == LG_QKV) a.tiles_n = (a.N + 2 * a.N2) / 256;
  a.k_splits = k_splits;
  if (EPI != LG_RESID && EPI != LG_QKV) a.k_per = a.K;
  const int items = a.tiles_m * a.tiles_n * k_splits;
  const int grid = items < t2_cus ? (items + 7) / 8 * 8 : t2_cus;   // one persistent workgroup per CU
  k_gemm_t256<EPI><<<grid, 256, T2_LDS, s>>>(a);
  return hipGetLastError();
}
static bool t2_usable(int M, int K) {
  static const int off = getenv("DLLM_NO_T256") ? 1 : 0;   // tuning aid
  return t2_ready && !off && M >= 256 && K % 32 == 0 && K >= 128;
}

template <int EPI>
static hipError_t lg_launch(hipStream_t s, LgArgs a, int k_splits = 1) {
  // 128-row tiles, two workgroups per CU (a 256-row form of this kernel, one workgroup per CU, measured
  // 2.3x slower: with a single wave per SIMD nothing covers its LDS and barrier waits)
  a.tiles_m = (a.M + 127) / 128;
  constexpr int tile_n = EPI == LG_SWIGLU ? LG_BN / 2 : LG_BN;
  a.tiles_n = (a.N + tile_n - 1) / tile_n;
  if constexpr (EPI == LG_QKV) {
    a.tiles_n1 = a.tiles_n;
    a.tiles_n2 = (a.N2 + LG_BN - 1) / LG_BN;
    a.tiles_n = a.tiles_n1 + 2 * a.tiles_n2;
  }
  const dim3 grid((a.tiles_m * a.tiles_n + 7) / 8 * 8, k_splits);
  k_gemm_mfma<128, EPI><<<grid, 256, 0, s>>>(a);
  return hipGetLastError();
}

// C[M,N] (=, +=) A[M,K] W[N,K]^T for bfloat16 operands; N % 4 == 0 and K % 8 == 0
hipError_t launch_gemm_mfma(hipStream_t s, const void* A, const void* W, void* C, int M, int N, int K, Epi epi) {
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)W; a.C = C; a.M = M; a.N = N; a.K = K;
  if (epi == EPI_STORE) return lg_launch<LG_STORE>(s, a);
  if (epi == EPI_STORE_F32) return lg_launch<LG_STORE_F32>(s, a);
  a.k_per = (K + LG_BK - 1) / LG_BK * LG_BK;
  return lg_launch<LG_RESID>(s, a);
}

// x[M,N] += A[M,K] W[N,K]^T with the sum over K split while that fills the chip better: split 0 adds
// into x, the others store their products for the next RMSNorm (or fold) to add, in split order.
hipError_t launch_gemm_resid_split(dllm_ctx* c, hipStream_t s, const void* A, const void* W, float* x, int M, int N, int K,
                                   int* n_delta) {
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)W; a.C = x; a.M = M; a.N = N; a.K = K;
  // short sums over few rows: the 128-row tiles fill the chip better
  const bool t2 = t2_usable(M, K) && (K >= 8192 || ((M + 255) / 256) * ((N + 255) / 256) >= 192);
  const int tiles = t2 ? ((M + 255) / 256) * ((N + 255) / 256) : ((M + 127) / 128) * ((N + LG_BN - 1) / LG_BN);
  int splits = (t2 ? 256 : 512) / tiles;                      // one 256-row workgroup or two 128-row ones fit a CU
  if (splits > LG_MAX_DELTA + 1) splits = LG_MAX_DELTA + 1;
  while (splits > 1 && K / splits < 512) --splits;
  if (splits < 1 || M > c->map.lg_delta_rows || N != c->cfg.d_model) splits = 1;
  a.k_per = ((K + splits - 1) / splits + LG_BK - 1) / LG_BK * LG_BK;
  splits = (K + a.k_per - 1) / a.k_per;
  a.delta = (float*)(c->ws + c->map.delta);
  a.delta_stride = c->map.lg_delta_stride;
  *n_delta = splits - 1;
  if (t2) return t2_launch<LG_RESID>(s, a, splits);
  return lg_launch<LG_RESID>(s, a, splits);
}

// The fused q/k/v product on 256-row tiles, its sum over K split to fill the chip: every split leaves
// [M, dq + 2 dkv] float partial sums (q | k | v) for the rotary kernel to add.  *n_part = 0: not taken.
hipError_t launch_gemm_qkv_split(dllm_ctx* c, hipStream_t s, const void* A, const void* Wq, const void* Wk, const void* Wv,
                                 int M, int dq, int dkv, int K, int* n_part) {
  *n_part = 0;
  if (!t2_usable(M, K) || M > c->map.qkvp_rows || dq % 256 != 0 || dkv % 256 != 0 || c->map.qkvp_stride == 0)
    return hipSuccess;
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)Wq; a.W2 = (const bf16_t*)Wk; a.W3 = (const bf16_t*)Wv;
  a.M = M; a.N = dq; a.N2 = dkv; a.K = K;
  const int tiles = ((M + 255) / 256) * ((dq + 2 * dkv) / 256);
  int splits = 256 / tiles;
  if (splits > LG_QKV_SPLITS) splits = LG_QKV_SPLITS;
  while (splits > 1 && K / splits < 1024) --splits;
  if (splits < 1 || M > c->map.lg_delta_rows) splits = 1;   // the split buffers cover lg_delta_rows rows
  if (tiles * splits < 128) return hipSuccess;            // too few work items: the 128-row tiles do better
  a.k_per = ((K + splits - 1) / splits + 31) / 32 * 32;
  splits = (K + a.k_per - 1) / a.k_per;
  a.delta = (float*)(c->ws + c->map.qkvp);
  a.delta_stride = c->map.qkvp_stride;
  *n_part = splits;
  return t2_launch<LG_QKV>(s, a, splits);
}

// q32[M,dq], k32[M,dkv] (float) and v[M,dkv] (bfloat16) = A[M,K] times the three projections, one launch
hipError_t launch_gemm_qkv(hipStream_t s, const void* A, const void* Wq, const void* Wk, const void* Wv, float* q32,
                           float* k32, void* v, int M, int dq, int dkv, int K) {
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)Wq; a.W2 = (const bf16_t*)Wk; a.W3 = (const bf16_t*)Wv;
  a.C = q32; a.C2 = k32; a.C3 = v;
  a.M = M; a.N = dq; a.N2 = dkv; a.K = K;
  return lg_launch<LG_QKV>(s, a);
}

// h[M,F] = silu(A Wg^T) * (A Wu^T), bfloat16 row-major
hipError_t launch_gemm_swiglu(hipStream_t s, const void* A, const void* Wg, const void* Wu, void* H, int M, int F,
                              int K) {
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)Wg; a.W2 = (const bf16_t*)Wu; a.C = H; a.M = M; a.N = F; a.K = K;
  if (t2_usable(M, K)) return t2_launch<LG_SWIGLU>(s, a);
  return lg_launch<LG_SWIGLU>(s, a);
}

// LM head on the compacted rows (row-major ws.xn) -> softmax statistics per 64 columns
hipError_t launch_gemm_lmstats(dllm_ctx* c, hipStream_t s, int max_rows, int* n_parts_out) {
  const dllm_config& f = c->cfg;
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = WSM(c, xn, bf16_t); a.W = (const bf16_t*)c->lm_head; a.M = max_rows; a.N = f.vocab; a.K = f.d_model;
  a.m_dev = WSM(c, status, int32_t) + 1;
  a.part = WSM(c, lm_part, float);
  a.n_parts = (f.vocab + 63) / 64;
  a.mask_id = f.mask_id;
  *n_parts_out = a.n_parts;
  if (t2_usable(max_rows, a.K)) return t2_launch<LG_LMSTATS>(s, a);
  return lg_launch<LG_LMSTATS>(s, a);
}

}  // namespace dllm
