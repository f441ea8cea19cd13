// bfloat16 matrix-core (MFMA) kernels for gfx950: GEMMs over many token rows.
#include "mfma_common.h"

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
  const float* rscale;     // optional [M]: A holds x * gain rounded to bfloat16; the row's normalisation factor
                           // multiplies the float accumulators (every epilogue but RESID, whose input is not a norm's)
  int M, N, K, tiles_m, tiles_n;
  float* tail;             // 256-row SWIGLU: scratch for the accumulators of K-split tail tiles, or nullptr
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
      const float rs = a.rscale ? a.rscale[m] : 1.0f;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int n = n0 + (wn >> 1) + i * 16 + 4 * g;
        f32x4 v = acc[0][i][j] * rs;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = v[e] / (1.0f + expf(-v[e])) * (acc[0][i + 2][j][e] * rs);
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
      const float rs = (a.rscale && m < M) ? a.rscale[m] : 1.0f;
      RowStat st;
      st.init();
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int n = n0 + wn + i * 16 + 4 * g + e;
          const float z = acc[0][i][j][e] * rs;
          if (n < N && n != a.mask_id) st.merge(z, n, 1.0f, z);
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
    const float rs = (EPI != LG_RESID && a.rscale) ? a.rscale[m] : 1.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = n0 + wn + i * 16 + 4 * g;
      f32x4 v = acc[0][i][j] * rs;
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

__device__ __forceinline__ void t2_copy16(const void* g, void* l) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)l, 16, 0, 0);
}

// The last, partly filled round of the persistent workgroups: when the tiles do not divide by the workgroups, the
// tiles of the last round are split along K so that every workgroup gets a share of them (at most T2_TAIL_SPLITS
// shares per tile); their accumulators go to scratch in register order and k_swiglu_tail adds the shares and applies
// the epilogue.  Derived from the device-resident row count, the same way in both kernels.
constexpr int T2_TAIL_SPLITS = 3, T2_TAIL_FLOATS = 256 * 256;
struct T2Tail { int n_full, n_tail, splits; };
__device__ __forceinline__ T2Tail t2_tail_plan(int n_tiles, int n_wg, bool enabled) {
  T2Tail t{n_tiles, 0, 1};
  if (!enabled || n_tiles <= n_wg) return t;
  const int nf = (n_tiles / n_wg) * n_wg, nt = n_tiles - nf;
  if (nt == 0) return t;
  int sp = n_wg / nt;
  sp = sp > T2_TAIL_SPLITS ? T2_TAIL_SPLITS : sp;
  if (sp < 2) return t;
  t.n_full = nf; t.n_tail = nt; t.splits = sp;
  return t;
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
  // two passes over the work items, each dealt the same way: the whole tiles (all K splits of the launch), then the
  // K shares of the tail tiles (SiLU*up launches with scratch only)
  const T2Tail tp = t2_tail_plan(n_tiles, gridDim.x, EPI == LG_SWIGLU && a.tail != nullptr);
  const int n_items_a = tp.n_full * a.k_splits, n_items_b = tp.n_tail * tp.splits;
  const int per_xcd_a = (n_items_a + 7) / 8, per_xcd_b = (n_items_b + 7) / 8;
  const int step = gridDim.x >> 3;
  const int iters_a = (per_xcd_a + step - 1) / step, iters_b = (per_xcd_b + step - 1) / step;
  for (int it = 0; it < iters_a + iters_b; ++it) {
  const bool is_tail = it >= iters_a;
  const int iw = (blockIdx.x >> 3) + (is_tail ? it - iters_a : it) * step;
  const int per_xcd = is_tail ? per_xcd_b : per_xcd_a;
  const int item = (blockIdx.x & 7) * per_xcd + iw;
  if (iw >= per_xcd || item >= (is_tail ? n_items_b : n_items_a)) continue;
  int split, tile;
  if (is_tail) { split = item / tp.n_tail; tile = tp.n_full + (item - split * tp.n_tail); }
  else { split = item / tp.n_full; tile = item - split * tp.n_full; }
  const int tn = tile / tiles_m, tm = tile - tn * tiles_m;
  const int m0 = tm * 256, n0 = tn * TILE_N;
  int k_begin = 0, k_end = K;
  if constexpr (EPI == LG_RESID || EPI == LG_QKV) {
    k_begin = split * a.k_per;
    k_end = k_begin + a.k_per < K ? k_begin + a.k_per : K;
  }
  if (is_tail) {
    const int per = ((K / 32) + tp.splits - 1) / tp.splits * 32;
    k_begin = split * per;
    k_end = k_begin + per < K ? k_begin + per : K;
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

  if (EPI == LG_SWIGLU && is_tail) {
    // a K share of a tail tile: the raw accumulators, in register order (a lane's 16 floats contiguous)
    float* dst = a.tail + ((int64_t)split * tp.n_tail + (tile - tp.n_full)) * T2_TAIL_FLOATS;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        f32x4* d = (f32x4*)(dst + ((((w * 4 + i) * 4 + j) * 64 + lane) << 4));
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4)
          d[e4] = f32x4{acc[i][j][e4 * 4], acc[i][j][e4 * 4 + 1], acc[i][j][e4 * 4 + 2], acc[i][j][e4 * 4 + 3]};
      }
    continue;
  }
  // lane holds token column l%32 of token tile j; features (e/4)*8 + (l/32)*4 + e%4 of weight tile i
  if constexpr (EPI == LG_LMSTATS) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + wm * 128 + j * 32 + r;
      const float rs = (a.rscale && m < M) ? a.rscale[m] : 1.0f;
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
            const float z = acc[i][j][e] * rs;
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
              const float z = acc[i][j][e] * rs;
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
    const float rs = (EPI != LG_RESID && a.rscale) ? a.rscale[m] : 1.0f;
    if constexpr (EPI == LG_SWIGLU) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int n = n0 + wn * 64 + i * 32 + e4 * 8 + h * 4;
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float gt = acc[i][j][e4 * 4 + e] * rs;
            v[e] = gt * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gt)) * (acc[i + 2][j][e4 * 4 + e] * rs);
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
              f32x4{acc[i][j][e4 * 4], acc[i][j][e4 * 4 + 1], acc[i][j][e4 * 4 + 2], acc[i][j][e4 * 4 + 3]} * rs;
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

// The K shares of the tail tiles of a SiLU(gate)*up launch of k_gemm_t256: one workgroup of 64 lanes per (tail tile,
// wave, gate tile i, token tile j) adds the shares in order, applies the row factor and the activation and stores the
// 32 x 32 outputs exactly as the fused epilogue would.
__global__ __launch_bounds__(64) void k_swiglu_tail(const LgArgs a, int n_wg) {
  int M = a.M;
  if (a.m_dev) { const int md = *a.m_dev; M = md < M ? md : M; }
  const int tiles_m = (M + 255) / 256;
  const T2Tail tp = t2_tail_plan(tiles_m * a.tiles_n, n_wg, true);
  const int tail = blockIdx.x >> 5, sub = blockIdx.x & 31;
  if (tail >= tp.n_tail) return;
  const int w = sub >> 3, i = (sub >> 2) & 1, j = sub & 3, lane = threadIdx.x;
  const int wm = w & 1, wn = w >> 1, r = lane & 31, h = lane >> 5;
  const int tile = tp.n_full + tail;
  const int tn = tile / tiles_m, tm = tile - tn * tiles_m;
  const int m = tm * 256 + wm * 128 + j * 32 + r;
  if (m >= M) return;
  const int N = a.N;
  float gt[16], up[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) { gt[e] = 0.f; up[e] = 0.f; }
  for (int sp = 0; sp < tp.splits; ++sp) {
    const float* src = a.tail + ((int64_t)sp * tp.n_tail + tail) * T2_TAIL_FLOATS;
    const f32x4* g4 = (const f32x4*)(src + ((((w * 4 + i) * 4 + j) * 64 + lane) << 4));
    const f32x4* u4 = (const f32x4*)(src + ((((w * 4 + i + 2) * 4 + j) * 64 + lane) << 4));
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      const f32x4 gv = g4[e4], uv = u4[e4];
#pragma unroll
      for (int e = 0; e < 4; ++e) { gt[e4 * 4 + e] += gv[e]; up[e4 * 4 + e] += uv[e]; }
    }
  }
  const float rs = a.rscale ? a.rscale[m] : 1.0f;
#pragma unroll
  for (int e4 = 0; e4 < 4; ++e4) {
    const int n = tn * 128 + wn * 64 + i * 32 + e4 * 8 + h * 4;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float gg = gt[e4 * 4 + e] * rs;
      v[e] = gg * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gg)) * (up[e4 * 4 + e] * rs);
    }
    if (n + 4 <= N) {
      *(uint2*)((bf16_t*)a.C + (int64_t)m * N + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    } else {
      for (int e = 0; e < 4 && n + e < N; ++e) ((bf16_t*)a.C)[(int64_t)m * N + n + e] = f32_to_bf16(v[e]);
    }
  }
}

// ------------------------------------------------------------------------------------------
// 65 .. 255 token rows (a few blocks in flight at small batch): the weights still have to stream from
// memory once and the products are few, so what counts is bytes in flight and how often the activations
// are re-read.  A workgroup of 4 waves owns 128 token rows x 64 weight rows; both operands are copied
// straight into a 4-stage LDS ring of 32-deep K stages (12 KiB each: three workgroups fit a CU), the
// activations are shared by the waves through LDS, the products are 32 x 32 x 16 ones (wave tile 64 x 32).
// Row swizzle and operand layout are those of the 256 x 256 kernel.  A wave's 32 weight rows are 16 gate
// rows followed by the 16 up rows of the same features for SiLU(gate)*up: both land in one lane.  The tile is
// 128 x 128 where the matrix is wide enough to still fill the chip (gate/up): fewer activation re-reads.
constexpr int TS_NS = 4;

template <int EPI, int WT>      // WT: 32-row weight tiles per wave (the workgroup's tile is 128 x 64*WT)
__global__ __launch_bounds__(256) void k_gemm_ts(const LgArgs a) {
  constexpr int BN = 64 * WT, TS_STAGE = 8192 + BN * 64;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[TS_NS * TS_STAGE];
  constexpr int TILE_N = (EPI == LG_SWIGLU) ? BN / 2 : BN;    // output features of a tile
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int M = a.M;
  if (a.m_dev) { const int md = *a.m_dev; M = md < M ? md : M; }
  const int N = a.N, K = a.K;
  const int tile = blockIdx.x;
  const int tn = tile / a.tiles_m, tm = tile - tn * a.tiles_m;
  const int m0 = tm * 128, n0 = tn * TILE_N;
  if (m0 >= M) return;
  const int wm = w & 1, wn = w >> 1;
  const int r = lane & 31, h = lane >> 5;
  int k_begin = 0, k_end = K;
  if constexpr (EPI == LG_RESID || EPI == LG_QKV) {
    k_begin = blockIdx.y * a.k_per;
    k_end = k_begin + a.k_per < K ? k_begin + a.k_per : K;
  }
  // copies: this wave moves token blocks 2w, 2w+1 (16 rows each) and weight blocks w*WT .. of a stage
  constexpr int NC = 2 + WT;
  const bf16_t* gsrc[NC];
#pragma unroll
  for (int q = 0; q < NC; ++q) {
    const int rr = (q < 2 ? (2 * w + q) : (w * WT + q - 2)) * 16 + (lane >> 2);
    const int piece = (lane & 3) ^ ((rr >> 2) & 3);
    if (q < 2) {
      int row = m0 + rr; row = row < M ? row : M - 1;
      gsrc[q] = a.A + (int64_t)row * K + piece * 8;
    } else if constexpr (EPI == LG_SWIGLU) {
      int row = n0 + (rr >> 5) * 16 + (rr & 15); row = row < N ? row : N - 1;     // every 32 rows: 16 gate, 16 up
      gsrc[q] = (((rr >> 4) & 1) ? a.W2 : a.W) + (int64_t)row * K + piece * 8;
    } else if constexpr (EPI == LG_QKV) {
      const int row = n0 + rr;                       // q | k | v stacked, each a multiple of 64 rows
      const bf16_t* wsel = row < N ? a.W : (row < N + a.N2 ? a.W2 : a.W3);
      const int lrow = row < N ? row : (row < N + a.N2 ? row - N : row - N - a.N2);
      gsrc[q] = wsel + (int64_t)lrow * K + piece * 8;
    } else {
      int row = n0 + rr; row = row < N ? row : N - 1;
      gsrc[q] = a.W + (int64_t)row * K + piece * 8;
    }
  }
  auto copy_stage = [&](int slot, int kd) {
    unsigned char* base = smem + slot * TS_STAGE;
    t2_copy16(gsrc[0] + kd, base + (2 * w) * 1024);
    t2_copy16(gsrc[1] + kd, base + (2 * w + 1) * 1024);
#pragma unroll
    for (int q = 0; q < WT; ++q) t2_copy16(gsrc[2 + q] + kd, base + 8192 + (w * WT + q) * 1024);
  };
  int offA[2], offW[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int slotp = ((2 * ks + h) ^ ((r >> 2) & 3)) * 16;
    offA[ks] = (wm * 64 + r) * 64 + slotp;
    offW[ks] = 8192 + (wn * 32 * WT + r) * 64 + slotp;
  }
  f32x16 acc[WT][2];   // [weight tile][token tile]
#pragma unroll
  for (int i = 0; i < WT; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int ns = (k_end - k_begin) / 32;      // K ranges are multiples of 32 (checked on the host)
#pragma unroll
  for (int st = 0; st < TS_NS - 1; ++st) copy_stage(st, k_begin + (st < ns ? st : ns - 1) * 32);
  for (int st = 0; st < ns; ++st) {
    // this wave's copies of stage st are the oldest of its NC * (NS - 1) outstanding ones
    __builtin_amdgcn_s_waitcnt(T2_VMCNT(NC * (TS_NS - 2)));
    __builtin_amdgcn_s_barrier();               // every wave's part of stage st is in; stage st - 1 is free
    {
      const int sn = st + TS_NS - 1;
      copy_stage(sn % TS_NS, k_begin + (sn < ns ? sn : ns - 1) * 32);   // past the end: a repeat into a free slot
    }
    const unsigned char* base = smem + (st % TS_NS) * TS_STAGE;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const u32x4 fa0 = *(const u32x4*)(base + offA[ks]), fa1 = *(const u32x4*)(base + offA[ks] + 2048);
#pragma unroll
      for (int i = 0; i < WT; ++i) {
        const u32x4 fw = *(const u32x4*)(base + offW[ks] + i * 2048);
        acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw), __builtin_bit_cast(bf16x8, fa0), acc[i][0], 0, 0, 0);
        acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw), __builtin_bit_cast(bf16x8, fa1), acc[i][1], 0, 0, 0);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(T2_VMCNT(0));   // the ring's trailing repeats must not outlive the workgroup

  // lane holds token column l%32 of token tile j; weight rows (e/4)*8 + (l/32)*4 + e%4 of the wave's tile
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int m = m0 + wm * 64 + j * 32 + r;
    if (m >= M) continue;
    const float rs = (EPI != LG_RESID && a.rscale) ? a.rscale[m] : 1.0f;
    if constexpr (EPI == LG_SWIGLU) {
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
      for (int e4 = 0; e4 < 2; ++e4) {
        const int n = n0 + (wn * WT + i) * 16 + e4 * 8 + h * 4;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float gt = acc[i][j][e4 * 4 + e] * rs;
          v[e] = gt * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * gt)) * (acc[i][j][8 + e4 * 4 + e] * rs);
        }
        if (n + 4 <= N) {
          *(uint2*)((bf16_t*)a.C + (int64_t)m * N + n) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        } else {
          for (int e = 0; e < 4 && n + e < N; ++e) ((bf16_t*)a.C)[(int64_t)m * N + n + e] = f32_to_bf16(v[e]);
        }
      }
    } else if constexpr (EPI == LG_QKV) {
      const int nt = N + 2 * a.N2;
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int n = n0 + (wn * WT + i) * 32 + e4 * 8 + h * 4;
        *(f32x4*)(a.delta + (int64_t)blockIdx.y * a.delta_stride + (int64_t)m * nt + n) =
            f32x4{acc[i][j][e4 * 4], acc[i][j][e4 * 4 + 1], acc[i][j][e4 * 4 + 2], acc[i][j][e4 * 4 + 3]} * rs;
      }
    } else {
#pragma unroll
      for (int i = 0; i < WT; ++i)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int n = n0 + (wn * WT + i) * 32 + e4 * 8 + h * 4;
        const f32x4 v = f32x4{acc[i][j][e4 * 4], acc[i][j][e4 * 4 + 1], acc[i][j][e4 * 4 + 2], acc[i][j][e4 * 4 + 3]};
        const int64_t at = (int64_t)m * N + n;
        if (n + 4 <= N) {
          if (blockIdx.y == 0) { f32x4* p = (f32x4*)((float*)a.C + at); *p = *p + v; }
          else *(f32x4*)(a.delta + (int64_t)(blockIdx.y - 1) * a.delta_stride + at) = v;
        } else {
          for (int e = 0; e < 4 && n + e < N; ++e) {
            if (blockIdx.y == 0) ((float*)a.C)[at + e] += v[e];
            else a.delta[(int64_t)(blockIdx.y - 1) * a.delta_stride + at + e] = v[e];
          }
        }
      }
    }
  }
}

template <int EPI, int WT>
static hipError_t ts_launch(hipStream_t s, LgArgs a, int k_splits = 1) {
  constexpr int bn = 64 * WT, tile_n = EPI == LG_SWIGLU ? bn / 2 : bn;
  a.tiles_m = (a.M + 127) / 128;
  a.tiles_n = EPI == LG_QKV ? (a.N + 2 * a.N2) / bn : (a.N + tile_n - 1) / tile_n;
  if (EPI != LG_RESID && EPI != LG_QKV) a.k_per = a.K;
  const dim3 grid(a.tiles_m * a.tiles_n, k_splits);
  k_gemm_ts<EPI, WT><<<grid, 256, 0, s>>>(a);
  return hipGetLastError();
}
// rows for which the streaming tiles are the better form: more than the weight-streaming kernels take, fewer
// than fill 256-row tiles
static bool ts_usable(int M, int K) {
  return M > 64 && M < 256 && K % 32 == 0 && K >= 128;
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
  return t2_ready && M >= 256 && K % 32 == 0 && K >= 128;
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
hipError_t launch_gemm_mfma(hipStream_t s, const void* A, const void* W, void* C, int M, int N, int K, Epi epi,
                            const float* rscale, const int32_t* m_dev) {
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)W; a.C = C; a.M = M; a.N = N; a.K = K;
  a.m_dev = m_dev;
  a.rscale = epi == EPI_RESID ? nullptr : rscale;
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
  a.m_dev = c->rows_dev;
  if (ts_usable(M, K) && M <= c->map.lg_delta_rows && N == c->cfg.d_model) {
    // streaming tiles: K split until about three workgroups per CU are in flight
    const int tiles = ((M + 127) / 128) * ((N + 63) / 64);
    int splits = 768 / tiles;
    if (splits > LG_MAX_DELTA + 1) splits = LG_MAX_DELTA + 1;
    while (splits > 1 && K / splits < 512) --splits;
    if (splits < 1) splits = 1;
    a.k_per = ((K + splits - 1) / splits + 31) / 32 * 32;
    splits = (K + a.k_per - 1) / a.k_per;
    a.delta = (float*)(c->ws + c->map.delta);
    a.delta_stride = c->map.lg_delta_stride;
    *n_delta = splits - 1;
    return ts_launch<LG_RESID, 1>(s, a, splits);
  }
  // short sums over few rows: the 128-row tiles fill the chip better, unless the 256-row tiles' K shares still are
  // long enough to pay for their fill and drain (measured at K = 4096: 5 row tiles, three shares of 1365, do; 4 row
  // tiles, four shares of 1024, do not)
  const int tiles256 = ((M + 255) / 256) * ((N + 255) / 256);
  int shares256 = tiles256 > 0 ? 256 / tiles256 : 1;
  shares256 = shares256 > LG_MAX_DELTA + 1 ? LG_MAX_DELTA + 1 : (shares256 < 1 ? 1 : shares256);
  const bool shares_pay = shares256 > 1 && K / shares256 >= 1280 && M <= c->map.lg_delta_rows && N == c->cfg.d_model;
  const bool t2 = t2_usable(M, K) && (K >= 8192 || tiles256 >= 192 || shares_pay);
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
  if (ts_usable(M, K) && M <= c->map.lg_delta_rows && dq % 64 == 0 && dkv % 64 == 0 && c->map.qkvp_stride > 0) {
    LgArgs a;
    memset(&a, 0, sizeof(a));
    a.A = (const bf16_t*)A; a.W = (const bf16_t*)Wq; a.W2 = (const bf16_t*)Wk; a.W3 = (const bf16_t*)Wv;
    a.M = M; a.N = dq; a.N2 = dkv; a.K = K;
    a.rscale = WSM(c, rscale, float);
    a.m_dev = c->rows_dev;
    const bool wide = dq % 128 == 0 && dkv % 128 == 0 && (dq + 2 * dkv) / 128 >= 64;   // 128 x 128 tiles still fill the chip
    const int tiles = ((M + 127) / 128) * ((dq + 2 * dkv) / (wide ? 128 : 64));
    int splits = 768 / tiles;
    if (splits > LG_QKV_SPLITS) splits = LG_QKV_SPLITS;
    while (splits > 1 && K / splits < 512) --splits;
    if (splits < 1) splits = 1;
    a.k_per = ((K + splits - 1) / splits + 31) / 32 * 32;
    splits = (K + a.k_per - 1) / a.k_per;
    a.delta = (float*)(c->ws + c->map.qkvp);
    a.delta_stride = c->map.qkvp_stride;
    *n_part = splits;
    if (wide) return ts_launch<LG_QKV, 2>(s, a, splits);
    return ts_launch<LG_QKV, 1>(s, a, splits);
  }
  if (!t2_usable(M, K) || M > c->map.qkvp_rows || dq % 256 != 0 || dkv % 256 != 0 || c->map.qkvp_stride == 0)
    return hipSuccess;
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)Wq; a.W2 = (const bf16_t*)Wk; a.W3 = (const bf16_t*)Wv;
  a.M = M; a.N = dq; a.N2 = dkv; a.K = K;
  a.rscale = WSM(c, rscale, float);
  a.m_dev = c->rows_dev;
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
                           float* k32, void* v, int M, int dq, int dkv, int K, const float* rscale,
                           const int32_t* m_dev) {
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.rscale = rscale;
  a.m_dev = m_dev;
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)Wq; a.W2 = (const bf16_t*)Wk; a.W3 = (const bf16_t*)Wv;
  a.C = q32; a.C2 = k32; a.C3 = v;
  a.M = M; a.N = dq; a.N2 = dkv; a.K = K;
  return lg_launch<LG_QKV>(s, a);
}

// h[M,F] = silu(A Wg^T) * (A Wu^T), bfloat16 row-major
hipError_t launch_gemm_swiglu(hipStream_t s, const void* A, const void* Wg, const void* Wu, void* H, int M, int F,
                              int K, const float* rscale, const int32_t* m_dev, float* tail, size_t tail_bytes) {
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.rscale = rscale;
  a.m_dev = m_dev;
  a.A = (const bf16_t*)A; a.W = (const bf16_t*)Wg; a.W2 = (const bf16_t*)Wu; a.C = H; a.M = M; a.N = F; a.K = K;
  if (ts_usable(M, K)) return ts_launch<LG_SWIGLU, 2>(s, a);
  if (t2_usable(M, K)) {
    // K-split tail tiles need scratch for one share per workgroup; worth it only if whole rounds come before them
    const int tiles = ((M + 255) / 256) * ((F + 127) / 128);
    const bool split_tail = tail != nullptr && tail_bytes >= (size_t)t2_cus * T2_TAIL_FLOATS * sizeof(float) &&
                            tiles > t2_cus && tiles % t2_cus != 0 && K >= 32 * 8 * T2_TAIL_SPLITS;
    a.tail = split_tail ? tail : nullptr;
    hipError_t e = t2_launch<LG_SWIGLU>(s, a);
    if (e != hipSuccess || !split_tail) return e;
    a.tiles_n = (F + 127) / 128;
    k_swiglu_tail<<<(t2_cus - 1) * 32, 64, 0, s>>>(a, t2_cus);
    return hipGetLastError();
  }
  return lg_launch<LG_SWIGLU>(s, a);
}

// LM head on the compacted rows (row-major ws.xn) -> softmax statistics per 64 columns
hipError_t launch_gemm_lmstats(dllm_ctx* c, hipStream_t s, int max_rows, int* n_parts_out) {
  const dllm_config& f = c->cfg;
  LgArgs a;
  memset(&a, 0, sizeof(a));
  a.A = WSM(c, xn, bf16_t); a.W = (const bf16_t*)c->lm_head; a.M = max_rows; a.N = f.vocab; a.K = f.d_model;
  a.m_dev = WSM(c, status, int32_t) + 1;
  a.rscale = WSM(c, rscale, float);
  a.part = WSM(c, lm_part, float);
  a.n_parts = (f.vocab + 63) / 64;
  a.mask_id = f.mask_id;
  *n_parts_out = a.n_parts;
  // (65 .. 255 rows stay on the 128 x 128 tiles: 4.3 TB/s at 128 rows, against 2.8 TB/s for the 128 x 64
  // streaming tiles, whose activation re-reads double the bytes the LM head moves)
  if (t2_usable(max_rows, a.K)) return t2_launch<LG_LMSTATS>(s, a);
  return lg_launch<LG_LMSTATS>(s, a);
}

// ------------------------------------------------------------------------------------------
// Probes for the benchmark: what this chip sustains on a plain stream read and on a loop of nothing but matrix
// instructions, measured in the same run as the kernels that are held against those figures.
__global__ __launch_bounds__(512) void k_probe_read(const u32x4* __restrict__ p, size_t n_vec, uint32_t* sink) {
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
  u32x4 acc = {0, 0, 0, 0};
  size_t i = tid;
  for (; i + 7 * stride < n_vec; i += 8 * stride) {      // eight 16-byte loads in flight per lane
    u32x4 t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= t[u];
  }
  for (; i < n_vec; i += stride) acc ^= p[i];
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = 1;   // keeps the loads alive
}

// one wave per SIMD, sixteen independent 32x32x16 bfloat16 products in flight, operands in registers
// random_bits: operands with random signs, mantissas and exponents 2^-9 .. 1 (the switching activity of real
// weights and activations) instead of values that share sign and exponent
__global__ __launch_bounds__(256) void k_probe_mfma(int iters, int random_bits, float* sink) {
  f32x16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  // operand bits that are ordinary finite bfloat16 values and differ from lane to lane and from tile to tile
  u32x4 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t s0 = 0x3f803f80u + (((threadIdx.x * 2654435761u) >> 20) & 0x007f007fu) + i * 0x00010001u;
    a[i] = u32x4{s0, s0 ^ 0x00100010u, s0 + 0x00020002u, s0 ^ 0x80008000u};
    b[i] = u32x4{s0 ^ 0x80000000u, s0 + 0x00030003u, s0 ^ 0x00008000u, s0 + 0x00040004u};
    if (random_bits) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        uint32_t hsh = (threadIdx.x * 8u + blockIdx.x * 2048u + i * 16u + e) * 2654435761u;
        hsh ^= hsh >> 15; hsh *= 2246822519u; hsh ^= hsh >> 13;
        // per 16-bit half: sign, exponent 118 + (0 .. 9), 7 mantissa bits
        const uint32_t lo = (hsh & 0x807fu) | ((118u + ((hsh >> 8) & 0xfu) % 10u) << 7);
        const uint32_t hi = ((hsh >> 16) & 0x807fu) | ((118u + ((hsh >> 24) & 0xfu) % 10u) << 7);
        const uint32_t v = lo | (hi << 16);
        if (e < 4) a[i][e] = v; else b[i][e - 4] = v;
      }
    }
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                                 __builtin_bit_cast(bf16x8, b[j]), acc[i * 4 + j], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) sum += acc[i][0] + acc[i][7];
  if (sum == 1.2345e-30f) sink[0] = sum;
}

hipError_t launch_probe_read(hipStream_t s, const void* buf, size_t bytes, void* sink) {
  k_probe_read<<<t2_cus * 2, 512, 0, s>>>((const u32x4*)buf, bytes / 16, (uint32_t*)sink);
  return hipGetLastError();
}

// flops of one launch: workgroups * 4 waves * iters * 16 products * 2*32*32*16
hipError_t launch_probe_mfma(hipStream_t s, int iters, int random_bits, void* sink, double* flops) {
  const int wgs = t2_cus;
  k_probe_mfma<<<wgs, 256, 0, s>>>(iters, random_bits, (float*)sink);
  *flops = (double)wgs * 4.0 * iters * 16.0 * 2.0 * 32 * 32 * 16;
  return hipGetLastError();
}

}  // namespace dllm
