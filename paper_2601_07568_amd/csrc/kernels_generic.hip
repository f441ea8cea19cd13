// Generic kernels of the denoise-step path: any shape, float or bfloat16 storage, scalar FMA
// arithmetic in float.  They are the whole path for float models and the fallback for bfloat16
// shapes the matrix-core kernels do not take; the small bookkeeping kernels (token map, rotary
// table, row compaction, statistics merge, unmask) are shared by both.
#include "common.h"
#include <math.h>

namespace dllm {


__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// block-wide reductions for blockDim.x <= 1024; red must hold 16 floats; result broadcast
__device__ inline float block_sum(float v, float* red) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float r = 0.f;
  for (int i = 0; i < nw; ++i) r += red[i];
  return r;
}
__device__ inline float block_max(float v, float* red) {
  v = wave_max(v);
  int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float r = -DEV_INF;
  for (int i = 0; i < nw; ++i) r = fmaxf(r, red[i]);
  return r;
}

// ------------------------------------------------------------------------------------------
// token map: sequence and position of every row of the forward
// Sequence lengths of a call, checked before anything addresses memory with them (one workgroup, first launch of
// every forward).  Steps: len_safe[b] = prefix_len[b] clamped to [0, max_len] (max_len = the host's max_prefix_len).
// Packed forwards: len_safe[0..B] = the cu_seqlens with every length clamped to [0, max_len] (max_len = the host's
// max_seqlen) and the total to T; cu_pad = the padded column offsets of the packed K/V scratch.  Any clamp, and a
// packed total different from T, sets DLLM_STATUS_BAD_LENGTH.  With a live count (steps only): the valid rows per
// sequence (q_valid[b] or Q for the live sequences b < n_live[0], -1 for the others: every row of theirs is padding
// and their attention is skipped) and the number of rows up to the last live sequence for the GEMMs that can skip rows.
// total_is_cap (packed forwards): T is only the capacity of the token buffer; the sequences may end before it, the
// rows behind them are padding (no position) and the row count goes to status[2] for the GEMMs that can skip rows.
__global__ void k_seq_check(int T, int B, int Q, int max_len, const int32_t* prefix_len, const int32_t* cu,
                            int32_t* len_safe, int32_t* cu_pad, const int32_t* q_valid, const int32_t* n_live,
                            int32_t* q_valid_eff, int32_t* status, int total_is_cap) {
  __shared__ int s_bad;
  if (threadIdx.x == 0) s_bad = 0;
  __syncthreads();
  if (Q > 0) {
    int nl = B;
    if (n_live) { nl = n_live[0]; nl = nl < 0 ? 0 : (nl > B ? B : nl); }
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
      const int p = prefix_len[b];
      const int pc = p < 0 ? 0 : (p > max_len ? max_len : p);
      if (pc != p && b < nl) s_bad = 1;
      len_safe[b] = pc;
      if (n_live) q_valid_eff[b] = b < nl ? (q_valid ? q_valid[b] : Q) : -1;
    }
    if (n_live && threadIdx.x == 0) status[2] = nl * Q;
  } else if (threadIdx.x == 0) {
    int acc = 0, pad = 0, bad = cu[0] != 0;
    len_safe[0] = 0;
    for (int b = 0; b < B; ++b) {
      int len = cu[b + 1] - cu[b];
      if (len < 0 || len > max_len) { bad = 1; len = len < 0 ? 0 : max_len; }
      if (acc + len > T) { bad = 1; len = T - acc; }
      cu_pad[b] = pad;
      acc += len;
      pad += (len + 31) / 32 * 32;
      len_safe[b + 1] = acc;
    }
    cu_pad[B] = pad;
    if (acc != T && !total_is_cap) bad = 1;
    if (total_is_cap) status[2] = acc;
    if (bad) s_bad = 1;
  }
  __syncthreads();
  if (threadIdx.x == 0 && s_bad) atomicOr(status, DLLM_STATUS_BAD_LENGTH);
}

// token map: sequence and position of every row of the forward, from the checked lengths.  Rows of a packed forward
// past the last sequence's end and padding rows of a step have no position (-1): nothing of theirs is cached or attended.
__global__ void k_token_map(int T, int B, int Q, const int32_t* len_safe, int32_t* tok_seq, int32_t* tok_pos,
                            const int32_t* q_valid) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  if (Q > 0) {
    int b = t / Q;
    tok_seq[t] = b;
    // padding rows of a step (past q_valid of their sequence; q_valid < 0: the whole sequence) have no position
    tok_pos[t] = (q_valid && (t - b * Q) >= q_valid[b]) ? -1 : len_safe[b] + (t - b * Q);
  } else {
    int lo = 0, hi = B;  // largest b with cu[b] <= t
    while (hi - lo > 1) {
      int mid = (lo + hi) >> 1;
      if (len_safe[mid] <= t) lo = mid; else hi = mid;
    }
    tok_seq[t] = lo;
    tok_pos[t] = t < len_safe[lo + 1] ? t - len_safe[lo] : -1;
  }
}

template <typename T>
__global__ void k_embed(int d, int vocab, const int32_t* tokens, const T* emb, float* x, int32_t* status) {
  int t = blockIdx.x;
  int tok = tokens[t];
  if (tok < 0 || tok >= vocab) {
    if (threadIdx.x == 0) atomicOr(status, DLLM_STATUS_BAD_TOKEN);
    tok = 0;
  }
  const T* row = emb + (int64_t)tok * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) x[(int64_t)t * d + i] = Elem<T>::load(row + i);
}

// cos/sin of position * base^(-2j/dh), evaluated in double so that long prefixes keep full
// float accuracy
__global__ void k_rope_table(int T, int half, double log2_base, const int32_t* tok_pos, float* cs, float* sn) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * half) return;
  int t = i / half, j = i - t * half;
  double theta = exp2(-(double)j / (double)half * log2_base);
  double a = (double)tok_pos[t] * theta;
  double s, c;
  sincos(a, &s, &c);
  cs[i] = (float)c;
  sn[i] = (float)s;
}

template <typename T>
__global__ void k_rmsnorm(int d, float eps, float* x, const T* gain, T* out, const int32_t* rows,
                          const int32_t* n_rows_dev, int frag_mt, const float* delta, int n_delta, int64_t delta_stride,
                          float* rscale, const int32_t* live_rows) {
  __shared__ float red[16];
  int r = blockIdx.x;
  if (live_rows && r >= *live_rows) return;
  int src = r;
  if (rows) {
    if (r >= *n_rows_dev) return;
    src = rows[r];
  }
  float* xr = x + (int64_t)src * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    float v = xr[i];
    if (n_delta > 0) {      // open K splits of the last residual projection, added in split order
      for (int sd = 0; sd < n_delta; ++sd) v += delta[sd * delta_stride + (int64_t)src * d + i];
      xr[i] = v;
    }
    ss += v * v;
  }
  ss = block_sum(ss, red);
  float rinv = 1.0f / sqrtf(ss / (float)d + eps);
  // rscale: the output is x * gain and the row factor goes to rscale[r] (the consuming GEMM multiplies its
  // accumulators by it); otherwise the output is the normalised row
  if (rscale) {
    if (threadIdx.x == 0) rscale[r] = rinv;
    rinv = 1.0f;
  }
  for (int i = threadIdx.x; i < d; i += blockDim.x) {   // a thread re-reads only what it wrote itself
    const int64_t at = frag_mt > 0 ? frag_offset(r, i, frag_mt) : (int64_t)r * d + i;
    Elem<T>::store(out + at, xr[i] * rinv * Elem<T>::load(gain + i));
  }
}

// ------------------------------------------------------------------------------------------
// C[M,N] = A[M,K] * W[N,K]^T, 64x64 tile, 16-deep slices through LDS, 4x4 per thread
template <typename T, int EPI>
__global__ __launch_bounds__(256) void k_gemm(const T* __restrict__ A, const T* __restrict__ W, void* Cv,
                                              int M, int N, int K, const float* rscale) {
  __shared__ float As[16][68];
  __shared__ float Ws[16][68];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int kk = k0 + lk + i;
      As[lk + i][lr] = (m0 + lr < M && kk < K) ? Elem<T>::load(A + (int64_t)(m0 + lr) * K + kk) : 0.f;
      Ws[lk + i][lr] = (n0 + lr < N && kk < K) ? Elem<T>::load(W + (int64_t)(n0 + lr) * K + kk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
    const float rs = (EPI != EPI_RESID && rscale) ? rscale[m] : 1.0f;   // row factor of a normalised input
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      int64_t idx = (int64_t)m * N + n;
      if (EPI == EPI_STORE) Elem<T>::store((T*)Cv + idx, acc[i][j] * rs);
      else if (EPI == EPI_STORE_F32) ((float*)Cv)[idx] = acc[i][j] * rs;
      else ((float*)Cv)[idx] += acc[i][j];
    }
  }
}

// ------------------------------------------------------------------------------------------
// rotary embedding of q and k (float projections in, one rounding to the storage type out), and
// K/V write into the paged pool (cached positions) and into the packed scratch (no-cache forward)
template <typename T>
__global__ void k_rope_kv(int Hq, int Hkv, int dh, const float* qf, const float* kf, T* q, const T* v,
                          const float* cs, const float* sn, const int32_t* tok_seq, const int32_t* tok_pos,
                          const int32_t* n_cache, T* pool_k, T* pool_v, KVView pool, T* pack_k, T* pack_v,
                          KVView pack, bool to_pack, int32_t* status, const float* part, int n_part,
                          int64_t part_stride) {
  const int t = blockIdx.x;
  const int half = dh >> 1;
  const float* c = cs + (int64_t)t * half;
  const float* s = sn + (int64_t)t * half;
  // n_part > 0: q, k, v arrive as n_part partial sums over K of one [T, Hq*dh + 2*Hkv*dh] float
  // matrix each (q | k | v); they are added in split order
  const int np = n_part > 0 ? n_part : 1;
  const int64_t ps = n_part > 0 ? part_stride : 0;
  const float* qs = n_part > 0 ? part + (int64_t)t * (Hq + 2 * Hkv) * dh : qf + (int64_t)t * Hq * dh;
  T* qt = q + (int64_t)t * Hq * dh;
  for (int i = threadIdx.x; i < Hq * half; i += blockDim.x) {
    int h = i / half, j = i - h * half;
    float a = 0.f, b = 0.f;
    for (int sp = 0; sp < np; ++sp) { a += qs[sp * ps + h * dh + j]; b += qs[sp * ps + h * dh + j + half]; }
    Elem<T>::store(qt + h * dh + j, a * c[j] - b * s[j]);
    Elem<T>::store(qt + h * dh + j + half, b * c[j] + a * s[j]);
  }
  const int b = tok_seq[t], pos = tok_pos[t];
  const bool cached = pos >= 0 && ((n_cache == nullptr) || (pos < n_cache[b]));   // pos < 0: a padding row
  const float* ks = n_part > 0 ? qs + Hq * dh : kf + (int64_t)t * Hkv * dh;
  const T* vt = v + (int64_t)t * Hkv * dh;
  const float* vparts = qs + (Hq + Hkv) * dh;
  for (int i = threadIdx.x; i < Hkv * half; i += blockDim.x) {
    int h = i / half, j = i - h * half;
    float a = 0.f, bb = 0.f;
    for (int sp = 0; sp < np; ++sp) { a += ks[sp * ps + h * dh + j]; bb += ks[sp * ps + h * dh + j + half]; }
    float r0 = a * c[j] - bb * s[j], r1 = bb * c[j] + a * s[j];
    int64_t ko, vo;
    int vs;
    if (cached) {
      if (kv_locate(pool, b, pos, h, ko, vo, vs)) {
        Elem<T>::store(pool_k + ko + j, r0);
        Elem<T>::store(pool_k + ko + j + half, r1);
      } else atomicOr(status, DLLM_STATUS_BAD_PAGE);
    }
    if (to_pack && pos >= 0) {
      kv_locate(pack, b, pos, h, ko, vo, vs);
      Elem<T>::store(pack_k + ko + j, r0);
      Elem<T>::store(pack_k + ko + j + half, r1);
    }
  }
  for (int i = threadIdx.x; i < Hkv * dh; i += blockDim.x) {
    int h = i / dh, j = i - h * dh;
    int64_t ko, vo;
    int vs;
    T val;
    if (n_part > 0) {
      float acc = 0.f;
      for (int sp = 0; sp < np; ++sp) acc += vparts[sp * ps + h * dh + j];
      Elem<T>::store(&val, acc);
    } else {
      val = vt[h * dh + j];
    }
    if (cached && kv_locate(pool, b, pos, h, ko, vo, vs)) pool_v[vo + (int64_t)j * vs] = val;
    if (to_pack && pos >= 0) {
      kv_locate(pack, b, pos, h, ko, vo, vs);
      pack_v[vo + (int64_t)j * vs] = val;
    }
  }
}

// The same for bfloat16 storage, eight token rows per workgroup: q and k are rotated four channel
// pairs per thread (vector loads and stores), and when the eight rows are eight consecutive, 8-aligned
// positions of one sequence their V values go out as one 16-byte store per channel (V is stored with the
// keys of a channel contiguous); otherwise row by row as above.
__global__ __launch_bounds__(256) void k_rope_kv8(int T, int Hq, int Hkv, int dh, const float* qf, const float* kf, bf16_t* q,
                                                  const bf16_t* v, const float* cs, const float* sn,
                                                  const int32_t* tok_seq, const int32_t* tok_pos, const int32_t* n_cache,
                                                  bf16_t* pool_k, bf16_t* pool_v, KVView pool, bf16_t* pack_k,
                                                  bf16_t* pack_v, KVView pack, bool to_pack, int32_t* status,
                                                  const float* part, int n_part, int64_t part_stride) {
  const int t0 = blockIdx.x * 8;
  const int tid = threadIdx.x + 256 * blockIdx.y, nthr = 256 * gridDim.y;   // gridDim.y workgroups share the eight rows' channels
  const int half = dh >> 1, hq4 = half >> 2;          // dh % 8 == 0
  const int np = n_part > 0 ? n_part : 1;
  const int64_t ps = n_part > 0 ? part_stride : 0;
  const int dq = Hq * dh, dkv = Hkv * dh, nt = dq + 2 * dkv;
  bool bad = false;
  __shared__ int s_b[8], s_pos[8], s_cached[8];
  if (threadIdx.x < 8) {
    const int t = t0 + threadIdx.x;
    int b = -1, pos = 0, cached = 0;
    if (t < T) {
      b = tok_seq[t]; pos = tok_pos[t];
      cached = pos >= 0 && ((n_cache == nullptr) || (pos < n_cache[b]));            // pos < 0: a padding row
    }
    s_b[threadIdx.x] = b; s_pos[threadIdx.x] = pos; s_cached[threadIdx.x] = cached;
  }
  __syncthreads();
  // q and k: all (row, head, 4-pair chunk) items of the eight rows in one flat loop, so that every
  // thread's loads are in flight together
  const int rows = T - t0 < 8 ? T - t0 : 8;
  const int nq = Hq * hq4, nk = Hkv * hq4;
  for (int idx = tid; idx < rows * (nq + nk); idx += nthr) {
    const int e = idx / (nq + nk), i = idx - e * (nq + nk);
    const int t = t0 + e;
    const bool is_q = i < nq;
    const int ii = is_q ? i : i - nq;
    const int h = ii / hq4, j4 = ii - h * hq4;
    const float4 c = ((const float4*)(cs + (int64_t)t * half))[j4], sn4 = ((const float4*)(sn + (int64_t)t * half))[j4];
    const float* src = n_part > 0 ? part + (int64_t)t * nt + (is_q ? 0 : dq) : (is_q ? qf + (int64_t)t * dq : kf + (int64_t)t * dkv);
    float4 a = {0.f, 0.f, 0.f, 0.f}, bb = {0.f, 0.f, 0.f, 0.f};
    for (int sp = 0; sp < np; ++sp) {
      const float4 x = *(const float4*)(src + sp * ps + h * dh + j4 * 4), y = *(const float4*)(src + sp * ps + h * dh + half + j4 * 4);
      a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w; bb.x += y.x; bb.y += y.y; bb.z += y.z; bb.w += y.w;
    }
    const uint2 lo = make_uint2(
        (uint32_t)f32_to_bf16(a.x * c.x - bb.x * sn4.x) | ((uint32_t)f32_to_bf16(a.y * c.y - bb.y * sn4.y) << 16),
        (uint32_t)f32_to_bf16(a.z * c.z - bb.z * sn4.z) | ((uint32_t)f32_to_bf16(a.w * c.w - bb.w * sn4.w) << 16));
    const uint2 hi = make_uint2(
        (uint32_t)f32_to_bf16(bb.x * c.x + a.x * sn4.x) | ((uint32_t)f32_to_bf16(bb.y * c.y + a.y * sn4.y) << 16),
        (uint32_t)f32_to_bf16(bb.z * c.z + a.z * sn4.z) | ((uint32_t)f32_to_bf16(bb.w * c.w + a.w * sn4.w) << 16));
    if (is_q) {
      bf16_t* qt = q + (int64_t)t * dq + h * dh;
      *(uint2*)(qt + j4 * 4) = lo;
      *(uint2*)(qt + half + j4 * 4) = hi;
      continue;
    }
    int64_t ko, vo;
    int vs;
    if (s_cached[e]) {
      if (kv_locate(pool, s_b[e], s_pos[e], h, ko, vo, vs)) {
        *(uint2*)(pool_k + ko + j4 * 4) = lo;
        *(uint2*)(pool_k + ko + half + j4 * 4) = hi;
      } else bad = true;
    }
    if (to_pack && s_pos[e] >= 0) {
      kv_locate(pack, s_b[e], s_pos[e], h, ko, vo, vs);
      *(uint2*)(pack_k + ko + j4 * 4) = lo;
      *(uint2*)(pack_k + ko + half + j4 * 4) = hi;
    }
  }
  // ---- V: eight rows of a channel at once where they are eight consecutive aligned positions
  bool group = t0 + 8 <= T && s_pos[0] >= 0 && (s_pos[0] & 7) == 0;
  for (int e = 1; e < 8 && group; ++e) group = s_b[e] == s_b[0] && s_pos[e] == s_pos[0] + e && s_cached[e] == s_cached[0];
  for (int i = tid; i < dkv; i += nthr) {
    const int h = i / dh, j = i - h * dh;
    bf16_t val[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int t = t0 + e;
      val[e] = 0;
      if (t >= T) continue;
      if (n_part > 0) {
        float acc = 0.f;
        for (int sp = 0; sp < np; ++sp) acc += part[(int64_t)t * nt + sp * ps + dq + dkv + i];
        val[e] = f32_to_bf16(acc);
      } else {
        val[e] = v[(int64_t)t * dkv + i];
      }
    }
    int64_t ko, vo;
    int vs;
    if (group) {
      const uint4 pk = make_uint4((uint32_t)val[0] | ((uint32_t)val[1] << 16), (uint32_t)val[2] | ((uint32_t)val[3] << 16),
                                  (uint32_t)val[4] | ((uint32_t)val[5] << 16), (uint32_t)val[6] | ((uint32_t)val[7] << 16));
      if (s_cached[0]) {
        if (kv_locate(pool, s_b[0], s_pos[0], h, ko, vo, vs)) *(uint4*)(pool_v + vo + (int64_t)j * vs) = pk;
        else bad = true;
      }
      if (to_pack) {
        kv_locate(pack, s_b[0], s_pos[0], h, ko, vo, vs);
        *(uint4*)(pack_v + vo + (int64_t)j * vs) = pk;
      }
    } else {
      for (int e = 0; e < 8 && t0 + e < T; ++e) {
        if (s_cached[e]) {
          if (kv_locate(pool, s_b[e], s_pos[e], h, ko, vo, vs)) pool_v[vo + (int64_t)j * vs] = val[e];
          else bad = true;
        }
        if (to_pack && s_pos[e] >= 0) {
          kv_locate(pack, s_b[e], s_pos[e], h, ko, vo, vs);
          pack_v[vo + (int64_t)j * vs] = val[e];
        }
      }
    }
  }
  if (bad) atomicOr(status, DLLM_STATUS_BAD_PAGE);
}

template <typename T>
__global__ void k_swiglu(int64_t n, const float* g, const float* u, T* h) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float x = g[i];
  Elem<T>::store(h + i, x / (1.0f + expf(-x)) * u[i]);
}

// ------------------------------------------------------------------------------------------
// attention, one workgroup per (row, query head): scores of a chunk of keys, running softmax,
// weighted sum of values.  No mask: every key of the row's sequence takes part.
constexpr int ATT_CHUNK = 1024;
template <typename T>
__global__ __launch_bounds__(256) void k_attention(int Hq, int dh, int Q, const T* q, T* o,
                                                   const int32_t* tok_seq, const int32_t* prefix_len,
                                                   const int32_t* cu, KVView kv, int32_t* status,
                                                   const int32_t* q_valid) {
  __shared__ float qs[128];
  __shared__ float sc[ATT_CHUNK];
  __shared__ int64_t offs[ATT_CHUNK];   // V offset of each key of the chunk, -1 = not addressable
  __shared__ float red[16];
  __shared__ float osum[256];
  const int t = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const int b = tok_seq[t];
  if (Q > 0 && q_valid && q_valid[b] < 0) return;      // the sequence is not part of this call
  const int kv_len = (Q > 0) ? prefix_len[b] + (q_valid ? min(max(q_valid[b], 0), Q) : Q) : cu[b + 1] - cu[b];
  const int kvh = h / (Hq / kv.n_kv_heads);
  const T* kbase = (const T*)kv.k;
  const T* vbase = (const T*)kv.v;
  if (tid < dh) qs[tid] = Elem<T>::load(q + ((int64_t)t * Hq + h) * dh + tid);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)dh);
  const int v_stride = kv.table ? kv.page_tokens : kv.tpad;
  const int ng = 256 / dh, grp = tid / dh, d = tid - grp * dh;
  float m = -DEV_INF, l = 0.f, oacc = 0.f;
  bool bad = false;
  for (int c0 = 0; c0 < kv_len; c0 += ATT_CHUNK) {
    const int n = min(ATT_CHUNK, kv_len - c0);
    float cm = -DEV_INF;
    for (int j = tid; j < n; j += 256) {
      int64_t ko, vo = -1;
      int vs;
      float s = -DEV_INF;
      if (kv_locate(kv, b, c0 + j, kvh, ko, vo, vs)) {
        const T* kr = kbase + ko;
        float a = 0.f;
        for (int e = 0; e < dh; ++e) a = fmaf(qs[e], Elem<T>::load(kr + e), a);
        s = a * scale;
      } else { bad = true; vo = -1; }
      sc[j] = s;
      offs[j] = vo;
      cm = fmaxf(cm, s);
    }
    cm = block_max(cm, red);
    if (cm == -DEV_INF) { __syncthreads(); continue; }
    const float m_new = fmaxf(m, cm);
    const float alpha = (m == -DEV_INF) ? 0.f : expf(m - m_new);
    float ps = 0.f;
    for (int j = tid; j < n; j += 256) {
      float p = (sc[j] == -DEV_INF) ? 0.f : expf(sc[j] - m_new);
      sc[j] = p;
      ps += p;
    }
    ps = block_sum(ps, red);   // has the barriers that publish sc[]
    l = l * alpha + ps;
    oacc *= alpha;
    if (grp < ng) {
      for (int j = grp; j < n; j += ng) {
        int64_t off = offs[j];
        if (off >= 0) oacc = fmaf(sc[j], Elem<T>::load(vbase + off + (int64_t)d * v_stride), oacc);
      }
    }
    m = m_new;
    __syncthreads();
  }
  osum[tid] = (grp < ng) ? oacc : 0.f;
  __syncthreads();
  if (tid < dh) {
    float tot = 0.f;
    for (int g2 = 0; g2 < ng; ++g2) tot += osum[g2 * dh + tid];
    Elem<T>::store(o + ((int64_t)t * Hq + h) * dh + tid, l > 0.f ? tot / l : 0.f);
  }
  if (bad) atomicOr(status, DLLM_STATUS_BAD_PAGE);
}

// ------------------------------------------------------------------------------------------
// Rows of the LM head: compacts, in ascending order, the rows whose token is the mask id (and,
// in a refresh call, whose position is not below n_commit), and writes the fixed outputs of
// the other eligible rows.  One workgroup of 1024 threads.
__global__ __launch_bounds__(1024) void k_mask_rows(int T, int32_t mask_id, int cap, const int32_t* tokens,
                                                    const int32_t* tok_seq, const int32_t* tok_pos,
                                                    const int32_t* n_commit, int32_t* rows, int32_t* status,
                                                    int32_t* cand, float* conf, float* entropy, int Q,
                                                    const int32_t* q_valid) {
  __shared__ int wcount[16];
  __shared__ int base_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) base_s = 0;
  __syncthreads();
  for (int c0 = 0; c0 < T; c0 += 1024) {
    const int t = c0 + tid;
    bool eligible = false, flag = false;
    if (t < T) {
      eligible = (n_commit == nullptr) || (tok_pos[t] >= n_commit[tok_seq[t]]);
      // padding rows of a step (past q_valid of their sequence) report their own token, whatever it is
      const bool pad = q_valid != nullptr && (t - tok_seq[t] * Q) >= q_valid[tok_seq[t]];
      flag = eligible && !pad && tokens[t] == mask_id;
      if (eligible && !flag) {
        cand[t] = tokens[t];
        conf[t] = 1.0f;
        if (entropy) entropy[t] = 0.f;
      }
    }
    const unsigned long long bal = __ballot(flag);
    const int lane_pre = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wcount[wave] = __popcll(bal);
    __syncthreads();
    int wave_pre = 0, total = 0;
    for (int w = 0; w < 16; ++w) { int cw = wcount[w]; if (w < wave) wave_pre += cw; total += cw; }
    const int base = base_s;
    if (flag) {
      int p = base + wave_pre + lane_pre;
      if (p < cap) rows[p] = t;
    }
    __syncthreads();
    if (tid == 0) base_s = base + total;
    __syncthreads();
  }
  if (tid == 0) {
    int n = base_s;
    if (n > cap) { atomicOr(status, DLLM_STATUS_ROWS_CAP); n = cap; }
    status[1] = n;
  }
}

// LM head on the compacted rows with the softmax statistics taken from the accumulators:
// each workgroup computes 64 rows x LM_TILE_N vocabulary columns in 64-column slices and keeps
// (max, argmax, sum exp, sum exp*z) per row.  The logits never leave the chip.
template <typename T>
__global__ __launch_bounds__(256) void k_lm_head(const T* __restrict__ A, const T* __restrict__ W, int V, int K,
                                                 int32_t mask_id, const int32_t* n_rows_dev, float* part,
                                                 int n_vtiles, const float* rscale) {
  __shared__ float As[16][68];
  __shared__ float Ws[16][68];
  __shared__ float Cs[64][65];
  const int M = *n_rows_dev;
  const int m0 = blockIdx.y * 64;
  if (m0 >= M) return;
  const int vt = blockIdx.x;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  RowStat st;
  st.init();
  for (int sub = 0; sub < LM_TILE_N / 64; ++sub) {
    const int n0 = vt * LM_TILE_N + sub * 64;
    if (n0 >= V) break;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int kk = k0 + lk + i;
        As[lk + i][lr] = (m0 + lr < M && kk < K) ? Elem<T>::load(A + (int64_t)(m0 + lr) * K + kk) : 0.f;
        Ws[lk + i][lr] = (n0 + lr < V && kk < K) ? Elem<T>::load(W + (int64_t)(n0 + lr) * K + kk) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < 16; ++kk) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) Cs[ty * 4 + i][tx * 4 + j] = acc[i][j];
    __syncthreads();
    if (tid < 64 && m0 + tid < M) {
      const float rs = rscale ? rscale[m0 + tid] : 1.0f;      // row factor of the normalised input
      for (int j = 0; j < 64; ++j) {
        int col = n0 + j;
        if (col < V && col != mask_id) st.push(Cs[tid][j] * rs, col);
      }
    }
    __syncthreads();
  }
  if (tid < 64 && m0 + tid < M) {
    float* p = part + ((int64_t)(m0 + tid) * n_vtiles + vt) * 4;
    p[0] = st.m;
    p[1] = __int_as_float(st.idx);
    p[2] = st.s;
    p[3] = st.t;
  }
}

// one wavefront per compacted row: merge the per-tile statistics and emit the outputs
__global__ __launch_bounds__(256) void k_lm_merge(const float* part, int n_vtiles, const int32_t* rows,
                                                  const int32_t* n_rows_dev, int32_t* cand, float* conf,
                                                  float* entropy, int by_token) {
  // 256 threads per row; a thread's partials are fetched eight at a time before they are merged, so the
  // loads of a batch are in flight together; lanes, then waves, merge in a fixed order
  __shared__ float4 wst[4];
  const int r = blockIdx.x;
  if (r >= *n_rows_dev) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float4* prow = (const float4*)part + (int64_t)(by_token ? rows[r] : r) * n_vtiles;
  RowStat st;
  st.init();
  for (int v0 = tid; v0 < n_vtiles; v0 += 256 * 8) {
    float4 p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int v = v0 + u * 256;
      p[u] = prow[v < n_vtiles ? v : n_vtiles - 1];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (v0 + u * 256 < n_vtiles) st.merge(p[u].x, __float_as_int(p[u].y), p[u].z, p[u].w);
  }
  for (int o = 1; o < 64; o <<= 1) {
    float m2 = __shfl_xor(st.m, o, 64), s2 = __shfl_xor(st.s, o, 64), t2 = __shfl_xor(st.t, o, 64);
    int i2 = __shfl_xor(st.idx, o, 64);
    st.merge(m2, i2, s2, t2);
  }
  if (lane == 0) wst[wave] = make_float4(st.m, __int_as_float(st.idx), st.s, st.t);
  __syncthreads();
  if (tid == 0) {
    st.init();
    for (int w = 0; w < 4; ++w) st.merge(wst[w].x, __float_as_int(wst[w].y), wst[w].z, wst[w].w);
    const int t = rows[r];
    cand[t] = st.idx;
    conf[t] = 1.0f / st.s;
    if (entropy) entropy[t] = (st.m + logf(st.s)) - st.t / st.s;
  }
}

// ------------------------------------------------------------------------------------------
// threshold + floor selection: one wavefront per (sequence, block)
__device__ inline bool conf_before(float a, int ia, float b, int ib) {
  // ordering "confidence descending, index ascending", NaN last
  bool an = (a != a), bn = (b != b);
  if (an != bn) return bn;
  if (!an && a != b) return a > b;
  return ia < ib;
}
__global__ __launch_bounds__(64) void k_unmask(int Q, int block_len, int32_t* q_tokens, const int32_t* cand,
                                               const float* conf, float thr, int min_unmask, int32_t mask_id,
                                               int32_t* n_unmasked, int32_t* n_remaining, int low_first,
                                               const int32_t* floors, int32_t* order, int32_t step_index) {
  // low_first: the statistic is an entropy - low values pass the threshold and come first; the
  // selection runs on its negation.  floors: optional floor per (sequence, block) instead of
  // min_unmask; a negative entry leaves the block untouched.
  __shared__ float cf[1024];
  __shared__ unsigned char msk[1024];
  const int nblk = Q / block_len;
  const int b = blockIdx.x / nblk, blk = blockIdx.x - b * nblk;
  const int64_t base = (int64_t)b * Q + (int64_t)blk * block_len;
  const int lane = threadIdx.x;
  int n_masked = 0;
  for (int i = lane; i < block_len; i += 64) {
    bool mk = q_tokens[base + i] == mask_id;
    msk[i] = mk;
    cf[i] = low_first ? -conf[base + i] : conf[base + i];
    n_masked += mk;
  }
  for (int o = 32; o > 0; o >>= 1) n_masked += __shfl_xor(n_masked, o, 64);
  __syncthreads();
  const int floor_in = floors ? floors[blockIdx.x] : min_unmask;
  const int floor_n = min(floor_in, n_masked);
  int n_un = 0;
  for (int i = lane; i < block_len; i += 64) {
    if (!msk[i] || floor_in < 0) continue;
    const float c = cf[i];
    bool take = (c >= thr);
    if (!take) {
      int rank = 0;
      for (int j = 0; j < block_len; ++j)
        if (msk[j] && j != i && conf_before(cf[j], j, c, i)) ++rank;
      take = rank < floor_n;
    }
    if (take) {
      q_tokens[base + i] = cand[base + i];
      if (order) order[base + i] = step_index;      // the decoding order of the trajectory being recorded
      ++n_un;
    }
  }
  for (int o = 32; o > 0; o >>= 1) n_un += __shfl_xor(n_un, o, 64);
  if (lane == 0) {
    if (n_unmasked) n_unmasked[blockIdx.x] = n_un;
    if (n_remaining) n_remaining[blockIdx.x] = n_masked - n_un;
  }
}

__global__ void k_copy_f32(const float* src, float* dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
__global__ void k_set_i32(int32_t* p, int n, int32_t v) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ==========================================================================================
// launchers
#define WS(c, field, type) ((type*)((c)->ws + (c)->map.field))
#define IS_BF16(c) ((c)->cfg.dtype == DLLM_BF16)

hipError_t launch_token_map(dllm_ctx* c, hipStream_t s, const StepGeom& g) {
  const bool live = g.Q > 0 && g.n_live != nullptr;
  k_seq_check<<<1, 256, 0, s>>>(g.T, g.B, g.Q, g.Q > 0 ? g.max_kv - g.Q : g.max_kv, g.prefix_len, g.cu_seqlens,
                                WS(c, len_safe, int32_t), WS(c, cu_pad, int32_t), g.Q > 0 ? g.q_valid : nullptr,
                                live ? g.n_live : nullptr, WS(c, q_valid_eff, int32_t), WS(c, status, int32_t),
                                g.Q == 0 && g.total_is_cap);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int32_t* qv = g.Q > 0 ? (live ? WS(c, q_valid_eff, int32_t) : g.q_valid) : nullptr;
  k_token_map<<<(g.T + 255) / 256, 256, 0, s>>>(g.T, g.B, g.Q, WS(c, len_safe, int32_t), WS(c, tok_seq, int32_t),
                                                WS(c, tok_pos, int32_t), qv);
  return hipGetLastError();
}

hipError_t launch_embed(dllm_ctx* c, hipStream_t s, const StepGeom& g) {
  const dllm_config& f = c->cfg;
  if (IS_BF16(c))
    k_embed<bf16_t><<<g.T, 256, 0, s>>>(f.d_model, f.vocab, g.tokens, (const bf16_t*)c->tok_emb,
                                        WS(c, x, float), WS(c, status, int32_t));
  else
    k_embed<float><<<g.T, 256, 0, s>>>(f.d_model, f.vocab, g.tokens, (const float*)c->tok_emb,
                                       WS(c, x, float), WS(c, status, int32_t));
  return hipGetLastError();
}

hipError_t launch_rope_table(dllm_ctx* c, hipStream_t s, const StepGeom& g) {
  const int half = c->cfg.head_dim / 2;
  const int n = g.T * half;
  k_rope_table<<<(n + 255) / 256, 256, 0, s>>>(g.T, half, log2((double)c->cfg.rope_base),
                                               WS(c, tok_pos, int32_t), WS(c, rope_cos, float),
                                               WS(c, rope_sin, float));
  return hipGetLastError();
}

// row-major bfloat16 output, four elements per thread and pass (d % 4 == 0)
__global__ __launch_bounds__(256) void k_rmsnorm_row4(int d, float eps, float* x, const bf16_t* gain, bf16_t* out,
                                                      const int32_t* rows, const int32_t* n_rows_dev, const float* delta,
                                                      int n_delta, int64_t delta_stride, float* rscale,
                                                      const int32_t* live_rows) {
  __shared__ float red[16];
  const int r = blockIdx.x;
  if (live_rows && r >= *live_rows) return;
  int src = r;
  if (rows) {
    if (r >= *n_rows_dev) return;
    src = rows[r];
  }
  float4* xr = (float4*)(x + (int64_t)src * d);
  const int n4 = d >> 2;
  float ss = 0.f;
  for (int i = threadIdx.x; i < n4; i += 256) {
    float4 v = xr[i];
    if (n_delta > 0) {      // open K splits of the last residual projection, added in split order
      for (int sd = 0; sd < n_delta; ++sd) {
        const float4 dv = ((const float4*)(delta + sd * delta_stride + (int64_t)src * d))[i];
        v.x += dv.x; v.y += dv.y; v.z += dv.z; v.w += dv.w;
      }
      xr[i] = v;
    }
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum(ss, red);
  // the output is x * gain; the row factor goes to rscale[r] and multiplies the consuming GEMM's accumulators
  if (threadIdx.x == 0) rscale[r] = 1.0f / sqrtf(ss / (float)d + eps);
  uint2* orow = (uint2*)(out + (int64_t)r * d);
  for (int i = threadIdx.x; i < n4; i += 256) {   // a thread re-reads only what it wrote itself
    const float4 v = xr[i];
    const uint2 gq = ((const uint2*)gain)[i];
    const float g0 = bf16_to_f32((bf16_t)(gq.x & 0xffff)), g1 = bf16_to_f32((bf16_t)(gq.x >> 16));
    const float g2 = bf16_to_f32((bf16_t)(gq.y & 0xffff)), g3 = bf16_to_f32((bf16_t)(gq.y >> 16));
    orow[i] = make_uint2((uint32_t)f32_to_bf16(v.x * g0) | ((uint32_t)f32_to_bf16(v.y * g1) << 16),
                         (uint32_t)f32_to_bf16(v.z * g2) | ((uint32_t)f32_to_bf16(v.w * g3) << 16));
  }
}

__global__ void k_fold_delta(int64_t n, float* x, const float* delta, int n_delta, int64_t delta_stride) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = x[i];
  for (int sd = 0; sd < n_delta; ++sd) v += delta[sd * delta_stride + i];
  x[i] = v;
}

hipError_t launch_fold_delta(dllm_ctx* c, hipStream_t s, int T, int n_delta, bool frag_path) {
  const int64_t n = (int64_t)T * c->cfg.d_model;
  k_fold_delta<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(n, WS(c, x, float), WS(c, delta, float), n_delta,
                                                          frag_path ? c->map.delta_stride : c->map.lg_delta_stride);
  return hipGetLastError();
}

// Row-major RMSNorm of the paths that launch one (large batches, no-cache forwards, float models).  bfloat16 models:
// the output is x * gain rounded to bfloat16 and the row factors go to ws.rscale (the consuming GEMMs multiply their
// float accumulators by them); float models: the output is the normalised row.
hipError_t launch_rmsnorm(dllm_ctx* c, hipStream_t s, const void* gain, int T, const int32_t* rows,
                          const int32_t* n_rows_dev, int frag_mt, int n_delta) {
  const dllm_config& f = c->cfg;
  if (IS_BF16(c) && f.d_model % 4 == 0)
    k_rmsnorm_row4<<<T, 256, 0, s>>>(f.d_model, f.rms_eps, WS(c, x, float), (const bf16_t*)gain, WS(c, xn, bf16_t), rows,
                                     n_rows_dev, WS(c, delta, float), n_delta, c->map.lg_delta_stride, WS(c, rscale, float),
                                     rows ? nullptr : c->rows_dev);
  else if (IS_BF16(c))
    k_rmsnorm<bf16_t><<<T, 256, 0, s>>>(f.d_model, f.rms_eps, WS(c, x, float), (const bf16_t*)gain,
                                        WS(c, xn, bf16_t), rows, n_rows_dev, 0, WS(c, delta, float), n_delta,
                                        c->map.lg_delta_stride, WS(c, rscale, float), rows ? nullptr : c->rows_dev);
  else
    k_rmsnorm<float><<<T, 256, 0, s>>>(f.d_model, f.rms_eps, WS(c, x, float), (const float*)gain,
                                       WS(c, xn, float), rows, n_rows_dev, 0, nullptr, 0, 0, nullptr,
                                       rows ? nullptr : c->rows_dev);
  return hipGetLastError();
}

template <typename T>
static void gemm_dispatch(hipStream_t s, const void* A, const void* W, void* C, int M, int N, int K, Epi epi,
                          const float* rscale) {
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  if (epi == EPI_STORE) k_gemm<T, EPI_STORE><<<grid, 256, 0, s>>>((const T*)A, (const T*)W, C, M, N, K, rscale);
  else if (epi == EPI_STORE_F32) k_gemm<T, EPI_STORE_F32><<<grid, 256, 0, s>>>((const T*)A, (const T*)W, C, M, N, K, rscale);
  else k_gemm<T, EPI_RESID><<<grid, 256, 0, s>>>((const T*)A, (const T*)W, C, M, N, K, nullptr);
}

hipError_t launch_gemm_generic(dllm_ctx* c, hipStream_t s, const void* A, const void* W, void* C, int M, int N,
                               int K, Epi epi, const float* rscale) {
  if (IS_BF16(c)) gemm_dispatch<bf16_t>(s, A, W, C, M, N, K, epi, rscale);
  else gemm_dispatch<float>(s, A, W, C, M, N, K, epi, nullptr);
  return hipGetLastError();
}

static KVView pool_view(dllm_ctx* c, const StepGeom& g, int layer) {
  const dllm_config& f = c->cfg;
  const size_t slab = kv_slab_elems(f) * elem_size(f);
  KVView kv;
  kv.k = c->kv_pool + (size_t)(layer * 2 + 0) * slab;
  kv.v = c->kv_pool + (size_t)(layer * 2 + 1) * slab;
  kv.table = g.block_table;
  kv.cu_pad = nullptr;
  kv.page_tokens = f.page_tokens;
  kv.max_pages = f.max_pages_per_seq;
  kv.n_pages = f.n_pages;
  kv.n_kv_heads = f.n_kv_heads;
  kv.head_dim = f.head_dim;
  kv.tpad = 0;
  return kv;
}

static KVView pack_view(dllm_ctx* c) {
  const dllm_config& f = c->cfg;
  KVView kv;
  kv.k = c->ws + c->map.kpack;
  kv.v = c->ws + c->map.vpack;
  kv.table = nullptr;
  kv.cu_pad = (const int32_t*)(c->ws + c->map.cu_pad);
  kv.page_tokens = 0;
  kv.max_pages = 0;
  kv.n_pages = 0;
  kv.n_kv_heads = f.n_kv_heads;
  kv.head_dim = f.head_dim;
  kv.tpad = (int32_t)c->map.tpad;
  return kv;
}

// keys/values a forward attends to: the paged pool in a denoise step, the packed scratch in a
// no-cache forward
KVView attention_view(dllm_ctx* c, const StepGeom& g, int layer) {
  return g.Q > 0 ? pool_view(c, g, layer) : pack_view(c);
}

hipError_t launch_rope_kv(dllm_ctx* c, hipStream_t s, const StepGeom& g, int layer, int n_part) {
  const dllm_config& f = c->cfg;
  KVView pool = pool_view(c, g, layer), pack = pack_view(c);
  const bool to_pack = g.Q == 0;
  const int32_t* n_cache = (g.Q > 0) ? nullptr : g.n_cache;
  // eight rows per workgroup; with few rows their channels are spread over up to 32 workgroups
  const int groups8 = (g.T + 7) / 8;
  int slices8 = groups8 >= 2048 ? 1 : (2048 + groups8 - 1) / groups8;
  if (slices8 > 32) slices8 = 32;
  if (IS_BF16(c) && f.head_dim % 8 == 0 && f.page_tokens % 8 == 0)
    k_rope_kv8<<<dim3(groups8, slices8), 256, 0, s>>>(g.T, f.n_q_heads, f.n_kv_heads, f.head_dim, WS(c, q32, float), WS(c, k32, float),
                                            WS(c, q, bf16_t), WS(c, v, bf16_t), WS(c, rope_cos, float),
                                            WS(c, rope_sin, float), WS(c, tok_seq, int32_t), WS(c, tok_pos, int32_t),
                                            n_cache, (bf16_t*)pool.k, (bf16_t*)pool.v, pool, (bf16_t*)pack.k,
                                            (bf16_t*)pack.v, pack, to_pack, WS(c, status, int32_t), WS(c, qkvp, float),
                                            n_part, c->map.qkvp_stride);
  else if (IS_BF16(c))
    k_rope_kv<bf16_t><<<g.T, 256, 0, s>>>(f.n_q_heads, f.n_kv_heads, f.head_dim, WS(c, q32, float), WS(c, k32, float),
                                          WS(c, q, bf16_t), WS(c, v, bf16_t), WS(c, rope_cos, float),
                                          WS(c, rope_sin, float), WS(c, tok_seq, int32_t), WS(c, tok_pos, int32_t),
                                          n_cache, (bf16_t*)pool.k, (bf16_t*)pool.v, pool, (bf16_t*)pack.k,
                                          (bf16_t*)pack.v, pack, to_pack, WS(c, status, int32_t), WS(c, qkvp, float),
                                          n_part, c->map.qkvp_stride);
  else
    k_rope_kv<float><<<g.T, 256, 0, s>>>(f.n_q_heads, f.n_kv_heads, f.head_dim, WS(c, q32, float), WS(c, k32, float),
                                         WS(c, q, float), WS(c, v, float), WS(c, rope_cos, float),
                                         WS(c, rope_sin, float), WS(c, tok_seq, int32_t), WS(c, tok_pos, int32_t),
                                         n_cache, (float*)pool.k, (float*)pool.v, pool, (float*)pack.k,
                                         (float*)pack.v, pack, to_pack, WS(c, status, int32_t), nullptr, 0, 0);
  return hipGetLastError();
}

hipError_t launch_swiglu(dllm_ctx* c, hipStream_t s, int T) {
  const int64_t n = (int64_t)T * c->cfg.d_ff;
  const unsigned grid = (unsigned)((n + 255) / 256);
  if (IS_BF16(c)) k_swiglu<bf16_t><<<grid, 256, 0, s>>>(n, WS(c, g, float), WS(c, u, float), WS(c, h, bf16_t));
  else k_swiglu<float><<<grid, 256, 0, s>>>(n, WS(c, g, float), WS(c, u, float), WS(c, h, float));
  return hipGetLastError();
}

hipError_t launch_attention_generic(dllm_ctx* c, hipStream_t s, const StepGeom& g, int layer) {
  const dllm_config& f = c->cfg;
  KVView kv = attention_view(c, g, layer);
  dim3 grid(g.T, f.n_q_heads);
  if (IS_BF16(c))
    k_attention<bf16_t><<<grid, 256, 0, s>>>(f.n_q_heads, f.head_dim, g.Q, WS(c, q, bf16_t), WS(c, o, bf16_t),
                                             WS(c, tok_seq, int32_t), g.prefix_len, g.cu_seqlens, kv,
                                             WS(c, status, int32_t), g.q_valid);
  else
    k_attention<float><<<grid, 256, 0, s>>>(f.n_q_heads, f.head_dim, g.Q, WS(c, q, float), WS(c, o, float),
                                            WS(c, tok_seq, int32_t), g.prefix_len, g.cu_seqlens, kv,
                                            WS(c, status, int32_t), g.q_valid);
  return hipGetLastError();
}

hipError_t launch_mask_rows(dllm_ctx* c, hipStream_t s, const StepGeom& g, int32_t* cand, float* conf,
                            float* entropy) {
  const int32_t* n_commit = (g.Q > 0) ? nullptr : g.n_cache;
  k_mask_rows<<<1, 1024, 0, s>>>(g.T, c->cfg.mask_id, (int)c->map.r_max, g.tokens, WS(c, tok_seq, int32_t),
                                 WS(c, tok_pos, int32_t), n_commit, WS(c, rows, int32_t),
                                 WS(c, status, int32_t), cand, conf, entropy, g.Q, g.Q > 0 ? g.q_valid : nullptr);
  return hipGetLastError();
}

hipError_t launch_lm_head_generic(dllm_ctx* c, hipStream_t s, int max_rows) {
  const dllm_config& f = c->cfg;
  dim3 grid(c->map.n_vtiles, (max_rows + 63) / 64);
  const int32_t* n_rows = WS(c, status, int32_t) + 1;
  if (IS_BF16(c))
    k_lm_head<bf16_t><<<grid, 256, 0, s>>>(WS(c, xn, bf16_t), (const bf16_t*)c->lm_head, f.vocab, f.d_model,
                                           f.mask_id, n_rows, WS(c, lm_part, float), c->map.n_vtiles,
                                           WS(c, rscale, float));
  else
    k_lm_head<float><<<grid, 256, 0, s>>>(WS(c, xn, float), (const float*)c->lm_head, f.vocab, f.d_model,
                                          f.mask_id, n_rows, WS(c, lm_part, float), c->map.n_vtiles, nullptr);
  return hipGetLastError();
}

hipError_t launch_lm_merge(dllm_ctx* c, hipStream_t s, int max_rows, int n_parts, int32_t* cand, float* conf,
                           float* entropy, bool by_token) {
  k_lm_merge<<<max_rows, 256, 0, s>>>(WS(c, lm_part, float), n_parts, WS(c, rows, int32_t),
                                     WS(c, status, int32_t) + 1, cand, conf, entropy, by_token ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_unmask(hipStream_t s, int B, int Q, int block_len, int32_t* q_tokens, const int32_t* cand,
                         const float* conf, float thr, int min_unmask, int32_t mask_id, int32_t* n_unmasked,
                         int32_t* n_remaining, bool low_first, const int32_t* floors, int32_t* order,
                         int32_t step_index) {
  k_unmask<<<B * (Q / block_len), 64, 0, s>>>(Q, block_len, q_tokens, cand, conf, low_first ? -thr : thr, min_unmask,
                                              mask_id, n_unmasked, n_remaining, low_first ? 1 : 0, floors, order,
                                              step_index);
  return hipGetLastError();
}

// Block states of multi-block decoding, one wave per sequence: count the unmasked positions of every
// block, then lane 0 walks the blocks in order and applies the transitions.  need_add / need_full are
// the unmasked counts that mean "10 %" and "95 %" complete (computed on the host in double).
__global__ __launch_bounds__(64) void k_fsm_update(int n_blocks, int block_len, const int32_t* gen, int32_t mask_id,
                                                   int32_t* state, int32_t* counter, int need_add, int need_full,
                                                   int delay, int nocache_round, int32_t* floor_next,
                                                   int32_t* summary) {
  __shared__ int filled[DLLM_FSM_MAX_BLOCKS];
  const int b = blockIdx.x, lane = threadIdx.x;
  const int32_t* g = gen + (int64_t)b * n_blocks * block_len;
  for (int k = 0; k < n_blocks; ++k) {
    int n = 0;
    for (int i = lane; i < block_len; i += 64) n += g[(int64_t)k * block_len + i] != mask_id;
    for (int o = 32; o > 0; o >>= 1) n += __shfl_xor(n, o, 64);
    if (lane == 0) filled[k] = n;
  }
  __syncthreads();
  if (lane != 0) return;
  int32_t* st = state + (int64_t)b * n_blocks;
  int32_t* ct = counter + (int64_t)b * n_blocks;
  if (nocache_round < 0) {      // derived: the round skipped the cache iff a block was stabilizing when it began
    nocache_round = 0;
    for (int k = 0; k < n_blocks; ++k) nocache_round |= st[k] == DLLM_BLOCK_STABILIZING;
  }
  for (int k = 0; k < n_blocks; ++k) {
    const int prev = k == 0 ? block_len : filled[k - 1];
    const int sk = st[k];
    if (sk == DLLM_BLOCK_STABILIZING) {
      if (nocache_round) ct[k] -= 1;
      if (ct[k] <= 0 && (k == 0 || st[k - 1] == DLLM_BLOCK_COMPLETED)) st[k] = DLLM_BLOCK_COMPLETED;
    } else if (sk == DLLM_BLOCK_ACTIVATED || sk == DLLM_BLOCK_FULLY_ACTIVATED) {
      if (filled[k] == block_len) { st[k] = DLLM_BLOCK_STABILIZING; ct[k] = delay; }
      else if (sk == DLLM_BLOCK_ACTIVATED && prev >= need_full) st[k] = DLLM_BLOCK_FULLY_ACTIVATED;
    } else if (sk == DLLM_BLOCK_INACTIVE) {
      if (k > 0 && st[k - 1] != DLLM_BLOCK_INACTIVE && prev >= need_add)
        st[k] = prev >= need_full ? DLLM_BLOCK_FULLY_ACTIVATED : DLLM_BLOCK_ACTIVATED;
      break;                                       // only the first inactive block can be added
    }
  }
  int lo = -1, hi = -1, stab = 0, done = 0;
  for (int k = 0; k < n_blocks; ++k) {
    const int sk = st[k];
    const bool act = sk == DLLM_BLOCK_ACTIVATED || sk == DLLM_BLOCK_FULLY_ACTIVATED;
    if (act) { if (lo < 0) lo = k; hi = k; }
    stab |= sk == DLLM_BLOCK_STABILIZING;
    done += sk == DLLM_BLOCK_COMPLETED;
    if (floor_next) floor_next[(int64_t)b * n_blocks + k] = sk == DLLM_BLOCK_FULLY_ACTIVATED ? 1 : (sk == DLLM_BLOCK_ACTIVATED ? 0 : -1);
  }
  if (summary) {
    summary[b * 4 + 0] = lo; summary[b * 4 + 1] = hi; summary[b * 4 + 2] = stab; summary[b * 4 + 3] = done;
  }
}

// The next round of every sequence from its block states: cached rounds since the last forward without cache, whether
// the next forward must skip the cache (a Stabilizing block, or the periodic refresh is due), and how many positions
// the cache holds after such a forward (prompt + the blocks Completed once its round's transitions are done).
__global__ void k_fsm_plan(int B, int n_blocks, int block_len, const int32_t* state, const int32_t* counter,
                           const int32_t* base_len, int refresh_every, int32_t* rounds_since, int32_t* nocache,
                           int32_t* n_commit_next) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int32_t* st = state + (int64_t)b * n_blocks;
  const int32_t* ct = counter + (int64_t)b * n_blocks;
  const int since = nocache[b] != 0 ? 0 : rounds_since[b] + 1;     // on entry nocache[b] tells how the round just done ran
  rounds_since[b] = since;
  bool stab = false;
  for (int k = 0; k < n_blocks; ++k) stab |= st[k] == DLLM_BLOCK_STABILIZING;
  int done = 0;
  for (int k = 0; k < n_blocks; ++k) {
    if (st[k] == DLLM_BLOCK_COMPLETED || (st[k] == DLLM_BLOCK_STABILIZING && ct[k] - 1 <= 0)) ++done;
    else break;
  }
  nocache[b] = (stab || (refresh_every > 0 && since >= refresh_every)) ? 1 : 0;
  n_commit_next[b] = (base_len ? base_len[b] : 0) + done * block_len;
}

hipError_t launch_fsm_plan(hipStream_t s, int B, int n_blocks, int block_len, const int32_t* state,
                           const int32_t* counter, const int32_t* base_len, int refresh_every, int32_t* rounds_since,
                           int32_t* nocache, int32_t* n_commit_next) {
  k_fsm_plan<<<(B + 63) / 64, 64, 0, s>>>(B, n_blocks, block_len, state, counter, base_len, refresh_every, rounds_since,
                                         nocache, n_commit_next);
  return hipGetLastError();
}

// Window of a cached round, per sequence: the run of active blocks (at most W), as the tokens, floors,
// prefix length and valid-row count that dllm_denoise_step_var / dllm_unmask_blocks take.  A sequence that
// has a stabilizing block (its round must not use the cache) or no active block gets an empty window.
// With the plan of the round (nocache != nullptr) every sequence that has an active block gets its window, whatever
// forward the round uses; q_valid_cached is the row count for the cached step (0 for the sequences the plan sends
// through the forward without cache).
__global__ void k_fsm_window(int n_blocks, int block_len, int W, const int32_t* gen, const int32_t* state,
                             const int32_t* base_len, int32_t pad_token, int32_t* win_tokens, int32_t* win_floor,
                             int32_t* prefix_len, int32_t* q_valid, int32_t* win_lo, const int32_t* nocache,
                             int32_t* q_valid_cached) {
  const int b = blockIdx.x;
  const int32_t* st = state + (int64_t)b * n_blocks;
  int lo = -1, hi = -1, stab = 0, done = 0;
  for (int k = 0; k < n_blocks; ++k) {
    const int sk = st[k];
    if (sk == DLLM_BLOCK_ACTIVATED || sk == DLLM_BLOCK_FULLY_ACTIVATED) { if (lo < 0) lo = k; hi = k; }
    stab |= sk == DLLM_BLOCK_STABILIZING;
    done += sk == DLLM_BLOCK_COMPLETED;
  }
  int nw = (lo < 0 || (stab && !nocache)) ? 0 : hi - lo + 1;
  if (nw > W) nw = W;
  if (nw == 0) lo = done;                              // an empty window sits right behind the cached blocks
  if (threadIdx.x == 0) {
    prefix_len[b] = base_len[b] + lo * block_len;
    q_valid[b] = nw * block_len;
    win_lo[b] = lo;
    if (q_valid_cached) q_valid_cached[b] = (nocache && nocache[b]) ? 0 : nw * block_len;
  }
  for (int k = threadIdx.x; k < W; k += blockDim.x) {
    const int sk = k < nw ? st[lo + k] : DLLM_BLOCK_INACTIVE;
    win_floor[(int64_t)b * W + k] = k < nw ? (sk == DLLM_BLOCK_FULLY_ACTIVATED ? 1 : (sk == DLLM_BLOCK_ACTIVATED ? 0 : -1)) : -1;
  }
  for (int j = threadIdx.x; j < W * block_len; j += blockDim.x)
    win_tokens[(int64_t)b * W * block_len + j] =
        j < nw * block_len ? gen[(int64_t)b * n_blocks * block_len + (int64_t)lo * block_len + j] : pad_token;
}
__global__ void k_fsm_scatter(int n_blocks, int block_len, int W, const int32_t* win_tokens, const int32_t* win_lo,
                              const int32_t* q_valid, int32_t* gen) {
  const int b = blockIdx.x;
  const int lo = win_lo[b], nv = q_valid[b];
  for (int j = threadIdx.x; j < nv; j += blockDim.x)
    gen[(int64_t)b * n_blocks * block_len + (int64_t)lo * block_len + j] = win_tokens[(int64_t)b * W * block_len + j];
}

hipError_t launch_fsm_window(hipStream_t s, int B, int n_blocks, int block_len, int W, const int32_t* gen,
                             const int32_t* state, const int32_t* base_len, int32_t pad_token, int32_t* win_tokens,
                             int32_t* win_floor, int32_t* prefix_len, int32_t* q_valid, int32_t* win_lo,
                             const int32_t* nocache, int32_t* q_valid_cached) {
  k_fsm_window<<<B, 256, 0, s>>>(n_blocks, block_len, W, gen, state, base_len, pad_token, win_tokens, win_floor,
                                 prefix_len, q_valid, win_lo, nocache, q_valid_cached);
  return hipGetLastError();
}

// The packed batch of a round's forward without cache: sequence b takes part iff the plan says so (nocache[b]) and it
// has an active block; its tokens are the prompt followed by the generation up to the end of its window.  One thread
// lays out the lengths (a sequence longer than max_seqlen, or one that does not fit the capacity any more, is left out
// with DLLM_STATUS_BAD_LENGTH), the grid then copies the tokens; rows behind the last sequence hold pad_token.
__global__ void k_fsm_pack_cu(int B, int n_blocks, int block_len, int W, int cap, int max_seqlen, const int32_t* state,
                              const int32_t* base_len, const int32_t* nocache, const int32_t* n_commit_plan,
                              int32_t* cu, int32_t* n_commit, int32_t* status) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int acc = 0, bad = 0;
  cu[0] = 0;
  for (int b = 0; b < B; ++b) {
    const int32_t* st = state + (int64_t)b * n_blocks;
    int lo = -1, hi = -1;
    for (int k = 0; k < n_blocks; ++k) {
      const int sk = st[k];
      if (sk == DLLM_BLOCK_ACTIVATED || sk == DLLM_BLOCK_FULLY_ACTIVATED) { if (lo < 0) lo = k; hi = k; }
    }
    if (lo >= 0 && hi - lo + 1 > W) hi = lo + W - 1;
    int len = 0;
    if (nocache[b] && lo >= 0) {
      const int base = base_len[b];
      const int64_t want = (int64_t)base + (int64_t)(hi + 1) * block_len;
      if (base < 0 || want > max_seqlen || acc + want > cap) bad = 1;
      else len = (int)want;
    }
    int nc = len > 0 ? n_commit_plan[b] : 0;
    if (nc < 0 || nc > len) { bad = 1; nc = nc < 0 ? 0 : len; }
    n_commit[b] = nc;
    acc += len;
    cu[b + 1] = acc;
  }
  if (bad) atomicOr(status, DLLM_STATUS_BAD_LENGTH);
}
__global__ void k_fsm_pack_tokens(int B, int n_blocks, int block_len, int max_prompt, int cap, const int32_t* cu,
                                  const int32_t* base_len, const int32_t* prompt, const int32_t* gen, int32_t pad_token,
                                  int32_t* out) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= cap) return;
  if (r >= cu[B]) { out[r] = pad_token; return; }
  int lo = 0, hi = B;                                  // largest b with cu[b] <= r (its sequence is not empty: r < cu[B])
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= r) lo = mid; else hi = mid;
  }
  const int i = r - cu[lo], base = base_len[lo];
  int32_t tok = pad_token;
  if (i < base) { if (i < max_prompt) tok = prompt[(int64_t)lo * max_prompt + i]; }
  else if (i - base < n_blocks * block_len) tok = gen[(int64_t)lo * n_blocks * block_len + (i - base)];
  out[r] = tok;
}
// The way back: the step outputs of such a forward, indexed by packed row, into the window layout [B, Q] of the
// sequences that took part (row j of sequence b's window is packed row cu[b] + prefix_len[b] + j).
__global__ void k_fsm_unpack(int Q, int cap, const int32_t* cu, const int32_t* prefix_len, const int32_t* q_valid,
                             const int32_t* nocache, const int32_t* src_cand, const float* src_conf, const float* src_ent,
                             int32_t* cand, float* conf, float* ent) {
  const int b = blockIdx.x;
  if (!nocache[b] || cu[b + 1] == cu[b]) return;
  int nv = q_valid[b];
  nv = nv < 0 ? 0 : (nv > Q ? Q : nv);
  const int64_t r0 = (int64_t)cu[b] + prefix_len[b];
  for (int j = threadIdx.x; j < nv; j += blockDim.x) {
    const int64_t r = r0 + j;
    if (r < 0 || r >= cu[b + 1] || r >= cap) continue;
    cand[(int64_t)b * Q + j] = src_cand[r];
    conf[(int64_t)b * Q + j] = src_conf[r];
    if (ent && src_ent) ent[(int64_t)b * Q + j] = src_ent[r];
  }
}
hipError_t launch_fsm_pack(hipStream_t s, int B, int n_blocks, int block_len, int W, int max_prompt, int cap,
                           int max_seqlen, const int32_t* state, const int32_t* base_len, const int32_t* nocache,
                           const int32_t* n_commit_plan, const int32_t* prompt, const int32_t* gen, int32_t pad_token,
                           int32_t* tokens, int32_t* cu, int32_t* n_commit, int32_t* status) {
  k_fsm_pack_cu<<<1, 64, 0, s>>>(B, n_blocks, block_len, W, cap, max_seqlen, state, base_len, nocache, n_commit_plan, cu,
                                 n_commit, status);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  k_fsm_pack_tokens<<<(cap + 255) / 256, 256, 0, s>>>(B, n_blocks, block_len, max_prompt, cap, cu, base_len, prompt, gen,
                                                      pad_token, tokens);
  return hipGetLastError();
}
hipError_t launch_fsm_unpack(hipStream_t s, int B, int Q, int cap, const int32_t* cu, const int32_t* prefix_len,
                             const int32_t* q_valid, const int32_t* nocache, const int32_t* src_cand,
                             const float* src_conf, const float* src_ent, int32_t* cand, float* conf, float* ent) {
  k_fsm_unpack<<<B, 256, 0, s>>>(Q, cap, cu, prefix_len, q_valid, nocache, src_cand, src_conf, src_ent, cand, conf, ent);
  return hipGetLastError();
}
hipError_t launch_fsm_scatter(hipStream_t s, int B, int n_blocks, int block_len, int W, const int32_t* win_tokens,
                              const int32_t* win_lo, const int32_t* q_valid, int32_t* gen) {
  k_fsm_scatter<<<B, 256, 0, s>>>(n_blocks, block_len, W, win_tokens, win_lo, q_valid, gen);
  return hipGetLastError();
}

hipError_t launch_fsm_update(hipStream_t s, int B, int n_blocks, int block_len, const int32_t* gen, int32_t mask_id,
                             int32_t* state, int32_t* counter, int need_add, int need_full, int delay, int nocache_round,
                             int32_t* floor_next, int32_t* summary) {
  k_fsm_update<<<B, 64, 0, s>>>(n_blocks, block_len, gen, mask_id, state, counter, need_add, need_full, delay,
                                nocache_round, floor_next, summary);
  return hipGetLastError();
}

// noisy sequence from a recorded decoding order: position j (0-based) keeps y if j < s, is masked if
// j >= s + k, and inside the window keeps y iff it was decoded by step s + kt
__global__ void k_noisy_sequence(int n, const int32_t* y, const int32_t* order, const int32_t* s_dev, int k, int kt,
                                 int32_t mask_id, int32_t* out) {
  const int b = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const int s = s_dev[b];
  const int64_t at = (int64_t)b * n + j;
  const int i = j + 1;
  int32_t v = y[at];
  if (i > s && (i > s + k || order[at] > s + kt)) v = mask_id;
  out[at] = v;
}

hipError_t launch_noisy_sequence(hipStream_t s, int B, int n, const int32_t* y, const int32_t* order, const int32_t* s_dev,
                                 int k, int kt, int32_t mask_id, int32_t* out) {
  dim3 grid((n + 255) / 256, B);
  k_noisy_sequence<<<grid, 256, 0, s>>>(n, y, order, s_dev, k, kt, mask_id, out);
  return hipGetLastError();
}

// early stop: one wave per sequence finds the first [MASK] and the first end-of-sequence token; the
// sequence is finished if the latter comes first.  A second, single-wave kernel lists the sequences
// that are not finished, in order.
__global__ __launch_bounds__(64) void k_eos_scan(int n, const int32_t* gen, int32_t eos_id, int32_t mask_id,
                                                 int32_t* finished, int32_t* first_eos) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int32_t* g = gen + (int64_t)b * n;
  int fm = n, fe = n;
  for (int i = lane; i < n; i += 64) {
    const int32_t t = g[i];
    if (t == mask_id && i < fm) fm = i;
    if (t == eos_id && i < fe) fe = i;
  }
  for (int o = 32; o > 0; o >>= 1) { fm = min(fm, __shfl_xor(fm, o, 64)); fe = min(fe, __shfl_xor(fe, o, 64)); }
  if (lane == 0) {
    const bool fin = fe < n && fe < fm;
    finished[b] = fin ? 1 : 0;
    if (first_eos) first_eos[b] = fin ? fe : -1;
  }
}
__global__ __launch_bounds__(64) void k_list_active(int B, const int32_t* finished, int32_t* active_index, int32_t* n_active) {
  const int lane = threadIdx.x;
  int count = 0;
  for (int b0 = 0; b0 < B; b0 += 64) {
    const int b = b0 + lane;
    const bool act = b < B && finished[b] == 0;
    const unsigned long long m = __builtin_amdgcn_ballot_w64(act);
    if (act) active_index[count + __popcll(m & ((1ull << lane) - 1ull))] = b;
    count += __popcll(m);
  }
  for (int b = count + lane; b < B; b += 64) active_index[b] = -1;
  if (lane == 0) n_active[0] = count;
}

hipError_t launch_eos_scan(hipStream_t s, int B, int n, const int32_t* gen, int32_t eos_id, int32_t mask_id,
                           int32_t* finished, int32_t* first_eos, int32_t* active_index, int32_t* n_active) {
  k_eos_scan<<<B, 64, 0, s>>>(n, gen, eos_id, mask_id, finished, first_eos);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !active_index || !n_active) return e;
  k_list_active<<<1, 64, 0, s>>>(B, finished, active_index, n_active);
  return hipGetLastError();
}

hipError_t launch_copy_f32(hipStream_t s, const float* src, float* dst, size_t n) {
  k_copy_f32<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(src, dst, n);
  return hipGetLastError();
}

// dst[i] = src[index[i]] for i < n_index (rows of row_len int32), the other rows of dst = fill; scatter: dst[index[i]]
// = src[i] for i < n_index.  Index values outside [0, B) address nothing (gather: the row is filled).
__global__ void k_gather_rows(int B, int row_len, const int32_t* index, const int32_t* n_index, const int32_t* src,
                              int32_t* dst, int32_t fill, int scatter) {
  const int i = blockIdx.x;
  int n = n_index[0];
  n = n < 0 ? 0 : (n > B ? B : n);
  const int j = i < n ? index[i] : -1;
  const bool ok = j >= 0 && j < B;
  if (scatter) {
    if (!ok) return;
    for (int e = threadIdx.x; e < row_len; e += blockDim.x) dst[(int64_t)j * row_len + e] = src[(int64_t)i * row_len + e];
  } else {
    for (int e = threadIdx.x; e < row_len; e += blockDim.x)
      dst[(int64_t)i * row_len + e] = ok ? src[(int64_t)j * row_len + e] : fill;
  }
}

hipError_t launch_gather_rows(hipStream_t s, int B, int row_len, const int32_t* index, const int32_t* n_index,
                              const int32_t* src, int32_t* dst, int32_t fill, bool scatter) {
  k_gather_rows<<<B, row_len >= 256 ? 256 : 64, 0, s>>>(B, row_len, index, n_index, src, dst, fill, scatter ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_set_i32(hipStream_t s, int32_t* p, int n, int32_t v) {
  k_set_i32<<<(n + 255) / 256, 256, 0, s>>>(p, n, v);
  return hipGetLastError();
}

}  // namespace dllm
