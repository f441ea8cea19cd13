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

enum SkEpi { SK_F32 = 1, SK_QKV = 2, SK_SWIGLU = 3, SK_LMSTATS = 4, SK_RESID = 5 };

struct SkArgs {
  const bf16_t* X;          // activations [M, K], fragment order
  const int32_t* n_lm_rows; // optional device count: the kernel does nothing if it is zero
  int M, K;
  const bf16_t* W0;         // main weight / Wq / W_gate / lm_head   (all in packed fragment order)
  const bf16_t* W1;         // Wk / W_up
  const bf16_t* W2;         // Wv
  int N0, N1, N2;           // rows of W0, W1, W2
  float* out_f32;           // F32: [M, N0]
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
  // Row scale of the activations (QKV, SWIGLU, LMSTATS, F32): X holds x * gain rounded to bfloat16, the row's
  // normalisation factor rsqrt(mean(x^2) + eps) is applied to the summed tile in float.  ss_in[row * ss_stride + p],
  // p < n_ss, are partial sums of squares of row `row` (added up in a fixed order); nullptr: no scale.
  const float* ss_in;
  int n_ss, ss_stride;
  float inv_d, eps;
  // RESID (residual projection x += X W0^T): a workgroup owns 16 columns for the whole of K, adds its tile to the
  // residual stream, writes x * gain_next in fragment order as the next GEMM's input and the rows' sums of squares
  // over its 16 columns to ss_out[row * ss_stride + workgroup].
  float* x;                 // residual stream [M, N0], in/out
  const bf16_t* gain_next;  // [N0]
  bf16_t* xg_out;           // fragment order, MT tiles
  float* ss_out;
  // LMSTATS
  float* part;              // [rows, n_parts, 4]
  int n_parts;
  int32_t mask_id;
};

constexpr int SK_KB = 128;  // k-elements per block: 4 matrix instructions deep
constexpr int SK_NW = 8;    // waves of a workgroup (they split K among themselves)
constexpr int SK_NW_RESID = 16;   // ... of a residual projection's (one 16-row weight tile per workgroup: the bytes in
                                  // flight come from the waves)

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
  // shorter stage keeps the registers of three stages within a wave's share
  constexpr int JB = (MT >= 3) ? 1 : 2;
  constexpr bool SCALED = (EPI != SK_RESID);
  constexpr int RPW = (MT * 16 + NW - 1) / NW;          // rows per wave when the row scales are summed
  __shared__ float red[NW][NT][MT][4][64];
  __shared__ float lmst[EPI == SK_LMSTATS ? MT : 1][4][16][4];
  __shared__ float rs[64];                              // row scale of the activations
  __shared__ float ssq[EPI == SK_RESID ? MT : 1][4][64];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int wg = blockIdx.x;
  const int K = a.K;
  const int M = a.M;
  if (a.n_lm_rows && *a.n_lm_rows <= 0) return;
  if (M <= 0) return;

  float xres = 0.f, gres = 0.f;                         // RESID: the thread's element of x and of the next gain

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
  if constexpr (EPI == SK_RESID) {
    // the element this thread will update (items beyond the first, with more than 1024 / 256 row tiles, load late)
    const int m = tid >> 8, iq = (tid >> 6) & 3;
    const int tok = m * 16 + c, n = row0[0] + 4 * g + iq;
    const bool ok = m < MT && tok < M && n < a.N0;
    xres = a.x[ok ? (int64_t)tok * a.N0 + n : 0];
    gres = bf16_to_f32(a.gain_next[ok ? n : 0]);
  }
  // QKV with one epilogue item per thread: what that item needs besides the sums - the row's position, its rotary
  // factors, the page of its cache slot - is requested now and arrives while the weights stream
  constexpr bool QKV_PRE = EPI == SK_QKV && MT * 256 <= NW * 64;
  float pcs = 0.f, psn = 0.f;
  int ppos = -1, ppage = -1;
  if constexpr (QKV_PRE) {
    const int m = tid >> 8, iq = (tid >> 6) & 3;
    const int tok = m * 16 + c;
    if (m < MT && tok < M) {
      ppos = a.tok_pos[tok];
      if (wg < a.n_q_wg + a.n_k_wg) {
        const int hj = row0[0] + 4 * g + iq;
        const int j = hj - (hj / a.dh) * a.dh;
        const int half = a.dh >> 1;
        pcs = a.rope_cos[(int64_t)tok * half + j];
        psn = a.rope_sin[(int64_t)tok * half + j];
      }
      const int pi = ppos >= 0 ? ppos / a.pool.page_tokens : a.pool.max_pages;
      if (pi < a.pool.max_pages) ppage = a.pool.table[(int64_t)a.tok_seq[tok] * a.pool.max_pages + pi];
    }
  }
  // kv_locate for that item from the values fetched above
  auto locate_pre = [&](int h, int64_t& k_off, int64_t& v_off, int& v_stride) -> bool {
    const KVView& kv = a.pool;
    if (ppos < 0 || ppage < 0 || ppage >= kv.n_pages) return false;
    const int slot = ppos - (ppos / kv.page_tokens) * kv.page_tokens;
    const int64_t ph = (int64_t)ppage * kv.n_kv_heads + h;
    k_off = (ph * kv.page_tokens + slot) * kv.head_dim;
    v_off = ph * kv.head_dim * kv.page_tokens + slot;
    v_stride = kv.page_tokens;
    return true;
  };

  f32x4 acc[NT][MT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[t][m] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Row scales: the wave adds up the partial sums of squares of rows w, w + NW, .. (one 16-byte load per lane covers
  // 256 partials of a row; lanes add their four, the wave adds its lanes in a fixed tree) and lane 0 keeps the
  // row's factor.  Called once the first weight stages are on their way: the partials come from the L2, the
  // weights from memory, so the wave waits no longer for them than it would for the weights alone.
  auto row_scales = [&]() {
    if constexpr (SCALED) {
      if (a.ss_in) {
        float4 ssv[RPW];
        const int idc = 4 * lane < a.ss_stride - 4 ? 4 * lane : a.ss_stride - 4;
#pragma unroll
        for (int q = 0; q < RPW; ++q) ssv[q] = *(const float4*)(a.ss_in + (int64_t)(w + q * NW) * a.ss_stride + idc);
#pragma unroll
        for (int q = 0; q < RPW; ++q) {
          const int row = w + q * NW;
          const int i0 = 4 * lane;
          float sq = (i0 < a.n_ss ? ssv[q].x : 0.f) + (i0 + 1 < a.n_ss ? ssv[q].y : 0.f) +
                     (i0 + 2 < a.n_ss ? ssv[q].z : 0.f) + (i0 + 3 < a.n_ss ? ssv[q].w : 0.f);
          for (int c0 = 256; c0 < a.n_ss; c0 += 256) {            // very wide models only
            const int i1 = c0 + 4 * lane;
            const int ic = i1 < a.ss_stride - 4 ? i1 : a.ss_stride - 4;
            const float4 v = *(const float4*)(a.ss_in + (int64_t)row * a.ss_stride + ic);
            sq += (i1 < a.n_ss ? v.x : 0.f) + (i1 + 1 < a.n_ss ? v.y : 0.f) + (i1 + 2 < a.n_ss ? v.z : 0.f) +
                  (i1 + 3 < a.n_ss ? v.w : 0.f);
          }
#pragma unroll
          for (int o = 1; o < 64; o <<= 1) sq += __shfl_xor(sq, o, 64);
          if (lane == 0 && row < 64) rs[row] = 1.0f / sqrtf(sq * a.inv_d + a.eps);
        }
      } else if (tid < 64) rs[tid] = 1.0f;
    }
  };

  // Software pipeline over this wave's stages (w, w+NW, ...): two stages are in flight while a third
  // is multiplied.  No load sits inside a branch of the steady-state loop (a branch around a load
  // makes the compiler wait for every outstanding load at the join); the drain is straight-line code.
  constexpr int SKB = JB * 32;                        // k-elements per stage
  const int n_full = K / SKB;                         // stages that need no tail guard
  const int ws = __builtin_amdgcn_readfirstlane(w);   // wave index as a scalar
  const int n_w = n_full > ws ? (n_full - ws + NW - 1) / NW : 0;
#define SK_LD(F, I) sk_load<NT, MT, JB, false>(F, wt, xf, ws + (I) * NW, g, K)
#define SK_MM(F) sk_mma<NT, MT, JB>(F, acc)
  if (n_w <= 1) {
    SkFrag<NT, MT, JB> f0;
    if (n_w == 1) SK_LD(f0, 0);
    row_scales();
    if (n_w == 1) SK_MM(f0);
  } else {
    SkFrag<NT, MT, JB> f0, f1, f2;
    SK_LD(f0, 0);
    SK_LD(f1, 1);
    row_scales();
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
  if (n_full * SKB < K && ws == n_full % NW) {   // ragged last stage
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

  if constexpr (EPI == SK_RESID) {
    // ---- residual projection: x += tile; next GEMM's input x * gain; sums of squares of the 16 columns per row
    static_assert(EPI != SK_RESID || NT == 1, "a residual projection's workgroup owns one 16-row weight tile");
    for (int item = tid; item < MT * 256; item += NW * 64) {
      const int m = item >> 8, iq = (item >> 6) & 3, ln = item & 63;
      const int tok = m * 16 + (ln & 15);
      const int n = row0[0] + 4 * (ln >> 4) + iq;
      float sum = 0.f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) sum += red[ww][0][m][iq][ln];
      float sq = 0.f;
      if (tok < M && n < a.N0) {
        const float v = (item == tid ? xres : a.x[(int64_t)tok * a.N0 + n]) + sum;
        const float gn = item == tid ? gres : bf16_to_f32(a.gain_next[n]);
        a.x[(int64_t)tok * a.N0 + n] = v;
        a.xg_out[frag_offset(tok, n, MT)] = f32_to_bf16(v * gn);
        sq = v * v;
      }
      ssq[m][iq][ln] = sq;
    }
    __syncthreads();
    if (tid < MT * 16) {          // the 16 contributions of a row (4 values of iq x 4 lane groups) in a fixed order
      const int m = tid >> 4, cc = tid & 15;
      float sq = 0.f;
#pragma unroll
      for (int iq = 0; iq < 4; ++iq)
#pragma unroll
        for (int lg = 0; lg < 4; ++lg) sq += ssq[m][iq][lg * 16 + cc];
      a.ss_out[(int64_t)tid * a.ss_stride + wg] = sq;
    }
    return;
  }

  for (int item = tid; item < MT * 256; item += NW * 64) {
    const int m = item >> 8, i = (item >> 6) & 3, ln = item & 63;
    const int tok = m * 16 + (ln & 15);
    const int fr = 4 * (ln >> 4) + i;          // row inside the 16-row tile
    float val[NT];
    const float rsc = SCALED ? rs[tok] : 1.0f;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      float s = 0.f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) s += red[ww][t][m][i][ln];
      val[t] = s * rsc;
    }
    const bool tok_ok = tok < M;
    if constexpr (EPI == SK_F32) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int n = row0[t] + fr;
        if (tok_ok && n < a.N0) a.out_f32[(int64_t)tok * a.N0 + n] = val[t];
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
          const float cs = QKV_PRE ? pcs : a.rope_cos[(int64_t)tok * half + j];
          const float sn = QKV_PRE ? psn : a.rope_sin[(int64_t)tok * half + j];
          const float v0 = val[0], v1 = val[1];
          const bf16_t r0 = f32_to_bf16(v0 * cs - v1 * sn), r1 = f32_to_bf16(v1 * cs + v0 * sn);
          if (isq) {
            a.out_bf16[(int64_t)tok * a.N0 + hj] = r0;
            a.out_bf16[(int64_t)tok * a.N0 + hj + half] = r1;
          } else {
            int64_t ko, vo;
            int vs;
            const int pos = QKV_PRE ? ppos : a.tok_pos[tok];
            if (pos < 0) {
              // a padding row: nothing of it is cached
            } else if (QKV_PRE ? locate_pre(h, ko, vo, vs) : kv_locate(a.pool, a.tok_seq[tok], pos, h, ko, vo, vs)) {
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
          const int pos = QKV_PRE ? ppos : a.tok_pos[tok];
          if (pos >= 0 && (QKV_PRE ? locate_pre(h, ko, vo, vs) : kv_locate(a.pool, a.tok_seq[tok], pos, h, ko, vo, vs)))
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

// partial sums of squares per row: one per 16-column tile of d_model; rows are ss_stride floats apart
static int sk_ss_stride(const dllm_ctx* c) { return ((c->cfg.d_model + 15) / 16 + 3) / 4 * 4; }

// Residual projection x += A * W^T: one workgroup of 16 waves per 16-column tile, the waves split K.  Its epilogue
// prepares the next GEMM's input (x * gain_next in fragment order, sums of squares per row): no RMSNorm launch.
// A workgroup re-reads all of A from the L2 (twice its weight bytes); that costs less than exchanging partial
// products between workgroups would (two memory round trips at the end of every launch).
hipError_t launch_sk_resid(dllm_ctx* c, hipStream_t s, const void* A, const void* W, int M, int N, int K,
                           const void* gain_next) {
  SkArgs a = sk_base(A, M, K);
  a.W0 = (const bf16_t*)W;   // packed
  a.N0 = N;
  a.x = WSM(c, x, float);
  a.gain_next = (const bf16_t*)gain_next;
  a.xg_out = WSM(c, xn, bf16_t);
  a.ss_out = WSM(c, ss, float);
  a.ss_stride = sk_ss_stride(c);
  return sk_launch_mt<1, SK_NW_RESID, SK_RESID>(s, a, (N + 15) / 16);
}

// the GEMM input comes with n_ss partial sums of squares per row
static void sk_row_scale(dllm_ctx* c, SkArgs& a, int n_ss) {
  a.ss_in = WSM(c, ss, float);
  a.n_ss = n_ss;
  a.ss_stride = sk_ss_stride(c);
  a.inv_d = 1.0f / (float)c->cfg.d_model;
  a.eps = c->cfg.rms_eps;
}

// Everything a denoise step of at most 64 rows needs before its first GEMM, in one launch of one workgroup per row:
// the checks of the device-resident lengths (workgroup 0 writes the clamped copies, the live-row count and the status
// bit, exactly as k_seq_check does; every workgroup derives its own sequence's values the same way), the row's
// sequence and position (k_token_map), its rotary table entries (k_rope_table) and its embedding: x[t] = E[token[t]] in float, x * gain of the first norm in
// fragment order as the first GEMM's input, the row's sum of squares as its single partial.
__global__ __launch_bounds__(256) void k_sk_prologue(int T, int B, int Q, int max_len, int d, int vocab, int mt, int half,
                                                     double log2_base, const int32_t* tokens, const int32_t* prefix_len,
                                                     const int32_t* q_valid, const int32_t* n_live, const bf16_t* emb,
                                                     const bf16_t* gain, float* x, bf16_t* xg, float* ss, int ss_stride,
                                                     int32_t* len_safe, int32_t* q_valid_eff, int32_t* tok_seq,
                                                     int32_t* tok_pos, float* cs, float* sn, int32_t* status,
                                                     int32_t mask_id, int cap, int32_t* rows, int32_t* cand, float* conf,
                                                     float* entropy) {
  __shared__ float red[4];
  __shared__ int s_bad;
  const int t = blockIdx.x;
  int nl = B;
  if (n_live) { nl = n_live[0]; nl = nl < 0 ? 0 : (nl > B ? B : nl); }
  if (t == 0) {
    if (threadIdx.x == 0) s_bad = 0;
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
      const int p = prefix_len[b];
      const int pc = p < 0 ? 0 : (p > max_len ? max_len : p);
      if (pc != p && b < nl) s_bad = 1;
      len_safe[b] = pc;
      if (n_live) q_valid_eff[b] = b < nl ? (q_valid ? q_valid[b] : Q) : -1;
    }
    if (n_live && threadIdx.x == 0) status[2] = nl * Q;
    __syncthreads();
    if (threadIdx.x == 0 && s_bad) atomicOr(status, DLLM_STATUS_BAD_LENGTH);
    // the rows of the LM head (k_mask_rows for a step of at most 64 rows: one wave, row r in lane r): the masked rows
    // that are not padding, in ascending order; every other row reports its own token with confidence 1
    if (cand && threadIdx.x < 64) {
      const int r = threadIdx.x;
      bool flag = false;
      if (r < T) {
        const int b2 = r / Q, j2 = r - b2 * Q;
        const bool hq = n_live != nullptr || q_valid != nullptr;
        const int qv2 = n_live ? (b2 < nl ? (q_valid ? q_valid[b2] : Q) : -1) : (q_valid ? q_valid[b2] : Q);
        const int tk = tokens[r];
        flag = !(hq && j2 >= qv2) && tk == mask_id;
        if (!flag) {
          cand[r] = tk;
          conf[r] = 1.0f;
          if (entropy) entropy[r] = 0.f;
        }
      }
      const unsigned long long bal = __ballot(flag);
      const int pre = __popcll(bal & ((1ull << r) - 1ull));
      if (flag && pre < cap) rows[pre] = r;
      if (r == 0) {
        int n = __popcll(bal);
        if (n > cap) { atomicOr(status, DLLM_STATUS_ROWS_CAP); n = cap; }
        status[1] = n;
      }
    }
  }
  // this row's sequence, position (padding rows have none) and rotary angles
  const int b = t / Q, jrow = t - b * Q;
  const int p = prefix_len[b];
  const int pc = p < 0 ? 0 : (p > max_len ? max_len : p);
  const bool have_qv = n_live != nullptr || q_valid != nullptr;
  const int qve = n_live ? (b < nl ? (q_valid ? q_valid[b] : Q) : -1) : (q_valid ? q_valid[b] : Q);
  const int pos = (have_qv && jrow >= qve) ? -1 : pc + jrow;
  if (threadIdx.x == 0) { tok_seq[t] = b; tok_pos[t] = pos; }
  for (int j = threadIdx.x; j < half; j += blockDim.x) {
    const double theta = exp2(-(double)j / (double)half * log2_base);
    const double ang = (double)pos * theta;
    double sv, cv;
    sincos(ang, &sv, &cv);
    cs[t * half + j] = (float)cv;
    sn[t * half + j] = (float)sv;
  }
  // embedding: x[t] = E[token[t]] (float), x * gain in fragment order, the row's sum of squares
  int tok = tokens[t];
  if (tok < 0 || tok >= vocab) {
    if (threadIdx.x == 0) atomicOr(status, DLLM_STATUS_BAD_TOKEN);
    tok = 0;
  }
  const bf16_t* row = emb + (int64_t)tok * d;
  float sq = 0.f;
  for (int u = threadIdx.x; u < (d >> 3); u += 256) {          // 16-byte units: 8 channels
    const uint4 ev = *(const uint4*)(row + 8 * u), gv = *(const uint4*)(gain + 8 * u);
    const uint32_t ew[4] = {ev.x, ev.y, ev.z, ev.w}, gw[4] = {gv.x, gv.y, gv.z, gv.w};
    float xv[8];
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      xv[2 * e] = __uint_as_float(ew[e] << 16);
      xv[2 * e + 1] = __uint_as_float(ew[e] & 0xffff0000u);
      o[e] = pack_bf16x2(xv[2 * e] * __uint_as_float(gw[e] << 16), xv[2 * e + 1] * __uint_as_float(gw[e] & 0xffff0000u));
      sq = fmaf(xv[2 * e], xv[2 * e], sq);
      sq = fmaf(xv[2 * e + 1], xv[2 * e + 1], sq);
    }
    float4* xr = (float4*)(x + (int64_t)t * d + 8 * u);
    xr[0] = make_float4(xv[0], xv[1], xv[2], xv[3]);
    xr[1] = make_float4(xv[4], xv[5], xv[6], xv[7]);
    *(uint4*)(xg + frag_offset(t, 8 * u, mt)) = make_uint4(o[0], o[1], o[2], o[3]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sq;
  __syncthreads();
  if (threadIdx.x == 0) ss[(int64_t)t * ss_stride] = (red[0] + red[1]) + (red[2] + red[3]);
}

hipError_t launch_sk_prologue(dllm_ctx* c, hipStream_t s, const StepGeom& g, const void* gain, int32_t* cand,
                              float* conf, float* entropy) {
  const dllm_config& f = c->cfg;
  const bool live = g.n_live != nullptr;
  k_sk_prologue<<<g.T, 256, 0, s>>>(g.T, g.B, g.Q, g.max_kv - g.Q, f.d_model, f.vocab, (g.T + 15) / 16, f.head_dim / 2,
                                    log2((double)f.rope_base), g.tokens, g.prefix_len, g.q_valid, live ? g.n_live : nullptr,
                                    (const bf16_t*)c->tok_emb, (const bf16_t*)gain, WSM(c, x, float), WSM(c, xn, bf16_t),
                                    WSM(c, ss, float), sk_ss_stride(c), WSM(c, len_safe, int32_t),
                                    WSM(c, q_valid_eff, int32_t), WSM(c, tok_seq, int32_t), WSM(c, tok_pos, int32_t),
                                    WSM(c, rope_cos, float), WSM(c, rope_sin, float), WSM(c, status, int32_t),
                                    f.mask_id, (int)c->map.r_max, WSM(c, rows, int32_t), cand, conf, entropy);
  return hipGetLastError();
}

// out[M,N] = A[M,K] * W[N,K]^T in float (debug logits)
hipError_t launch_sk_f32(dllm_ctx* c, hipStream_t s, const void* A, const void* W, float* out, int M, int N, int K,
                         int n_ss) {
  SkArgs a = sk_base(A, M, K);
  sk_row_scale(c, a, n_ss);
  a.W0 = (const bf16_t*)W;
  a.N0 = N;
  a.out_f32 = out;
  return sk_launch_mt<4, 4, SK_F32>(s, a, (N + 63) / 64);
}

// fused q/k/v projection of a denoise step: rotary embedding on q and k, q to the workspace,
// k and v into the in-flight pages of the pool
hipError_t launch_sk_qkv(dllm_ctx* c, hipStream_t s, const StepGeom& g, int layer, const KVView& pool, int n_ss) {
  const dllm_config& f = c->cfg;
  SkArgs a = sk_base(c->ws + c->map.xn, g.T, f.d_model);
  sk_row_scale(c, a, n_ss);
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
hipError_t launch_sk_swiglu(dllm_ctx* c, hipStream_t s, int layer, int M, int n_ss) {
  const dllm_config& f = c->cfg;
  SkArgs a = sk_base(c->ws + c->map.xn, M, f.d_model);
  sk_row_scale(c, a, n_ss);
  const dllm_layer_w& P = c->packed_layers[layer];
  a.W0 = (const bf16_t*)P.w_gate; a.W1 = (const bf16_t*)P.w_up;
  a.N0 = f.d_ff;
  a.out_bf16 = WSM(c, h, bf16_t);
  // (three tile pairs per workgroup -- 256 equal workgroups at F = 12288, a third of the activation reads --
  // measured no faster than one: 40.8 against 41.7 us)
  return sk_launch_mt<2, SK_NW, SK_SWIGLU>(s, a, (f.d_ff + 15) / 16);
}

// LM head on all rows of the step (ws.xn holds x * final gain) -> per-64-column softmax statistics of every row;
// the merge picks the masked ones.  If no row is masked (device count) nothing is computed.
hipError_t launch_sk_lmstats(dllm_ctx* c, hipStream_t s, int T, int n_ss, int* n_parts_out) {
  const dllm_config& f = c->cfg;
  SkArgs a = sk_base(c->ws + c->map.xn, T, f.d_model);
  sk_row_scale(c, a, n_ss);
  a.n_lm_rows = WSM(c, status, int32_t) + 1;
  a.W0 = (const bf16_t*)c->packed_lm_head;
  a.N0 = f.vocab;
  a.part = WSM(c, lm_part, float);
  a.n_parts = (f.vocab + 63) / 64;
  a.mask_id = f.mask_id;
  *n_parts_out = a.n_parts;
  return sk_launch_mt<4, 4, SK_LMSTATS>(s, a, a.n_parts);
}

}  // namespace dllm
