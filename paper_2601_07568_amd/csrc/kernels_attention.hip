// bfloat16 matrix-core (MFMA) kernels for gfx950: attention.
#include "mfma_common.h"

namespace dllm {

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
  int pg_cap;               // k_attn_dl: page ids of a sequence that its LDS copy of the block table holds
  float scale_log2;         // log2(e) / sqrt(DH)
  float* part_o;            // [T*Hq, n_units, DH]
  float* part_ml;           // [T*Hq, n_units, 2]
  int32_t* status;
};


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
    mx = rows_max(mx);
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
  if (paged && a.q_valid && a.q_valid[b] < 0) return;       // the sequence is not part of this call
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
  if (paged && pt % 32 == 0) {
    // A 32-key block lies inside one page, so its page id does not depend on where the sequence ends: the ids of a
    // wave's first two blocks are requested before the sequence length is known (the table row has max_pages
    // entries whatever the length), one memory round trip less in front of the K/V loads; later pairs' ids are
    // requested a pair ahead.
    auto block_page = [&](int kb, int (&pg)[3]) {
      const int pi = (kb << 5) / pt;
      const int v = table[pi < kv.max_pages ? pi : kv.max_pages - 1];
      pg[0] = pg[1] = pg[2] = pi < kv.max_pages ? v : -1;
    };
    int pga[3], pgb[3];
    block_page(unit, pga);
    block_page(unit + a.n_units, pgb);
    for (int kb = unit; kb < nkb; kb += 2 * a.n_units) {
      const int kb2 = kb + a.n_units;
      const bool two = kb2 < nkb;
      Blk ba, bb;
      issue(kb, pga, ba);
      if (two) issue(kb2, pgb, bb);
      else issue(kb, pga, bb);                    // a repeat of the first block's loads: no branch around a load
      block_page(kb + 2 * a.n_units, pga);
      block_page(kb2 + 2 * a.n_units, pgb);
      compute(kb, ba);
      if (two) compute(kb2, bb);
    }
  } else {
    for (int kb = unit; kb < nkb; kb += 2 * a.n_units) {
      const int kb2 = kb + a.n_units;
      const bool two = kb2 < nkb;
      const int kbb = two ? kb2 : kb;             // a repeat of the first block's loads: no branch around a load
      int pga[3], pgb[3];
      pages(kb, pga);
      pages(kbb, pgb);
      Blk ba, bb;
      issue(kb, pga, ba);
      issue(kbb, pgb, bb);
      compute(kb, ba);
      if (two) compute(kb2, bb);
    }
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
  if (n_units == 2) {                                   // the common case at large batch: no padded chunk of eight
    const int64_t slot = row * 2;
    const float4 ml = *(const float4*)(part_ml + slot * 2);            // (m0, l0, m1, l1)
    const float o0 = part_o[slot * DH + d], o1 = part_o[(slot + 1) * DH + d];
    const float Mn = fmaxf(ml.x, ml.z);
    if (Mn > -DEV_INF) {
      const float s0 = exp2f(ml.x - Mn), s1 = exp2f(ml.z - Mn);
      den = fmaf(ml.w, s1, ml.y * s0);
      num = fmaf(o1, s1, o0 * s0);
    }
  } else
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
  if (PAGED && a.q_valid && a.q_valid[b] < 0) return;        // the sequence is not part of this call
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

  // One 64-key block.  The waves of a workgroup leave the block's barrier in the same phase, so the
  // pipes (LDS, matrix, vector) only overlap where one wave's instruction order lets them: all K
  // fragments of the block are requested first, the scores of both 32-key halves are issued back to
  // back, and each half's V^T fragments are requested before its softmax (vector arithmetic, no LDS: its
  // reductions are row swaps), which runs while the matrix pipe still works on the other half.  A half beyond the sequence is multiplied like any
  // other: its scores are masked to -inf (the running maximum is finite after the first half) and its
  // V^T columns are zero in LDS.
  auto compute = [&](int buf, int kb64) {
    const int k0 = kb64 << 6;
    const int lk = lane ^ (4 * g);
    u32x4 kf[2][2][KK];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[half][tt][kk] = sk[buf][half][tt][kk][lk ^ kk];
    __builtin_amdgcn_sched_barrier(0);
    f32x4 s[2][2][QT];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
        for (int t = 0; t < QT; ++t) s[half][tt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
          for (int t = 0; t < QT; ++t) s[half][tt][t] = mfma16(kf[half][tt][kk], qf[t][kk], s[half][tt][t]);
      }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      u32x4 vf[DT];
#pragma unroll
      for (int d = 0; d < DT; ++d) vf[d] = sv[buf][half][d][lk ^ (2 * half)];
      __builtin_amdgcn_sched_barrier(0);
      u32x4 pf[QT], pl[QT];
      attn_softmax_block<DT, QT>(s[half], k0 + half * 32, kv_len, g, a.scale_log2, m_run, l_run, oacc, pf, pl);
#pragma unroll
      for (int d = 0; d < DT; ++d) {
#pragma unroll
        for (int t = 0; t < QT; ++t) oacc[d][t] = mfma16(vf[d], pf[t], oacc[d][t]);
#pragma unroll
        for (int t = 0; t < QT; ++t) oacc[d][t] = mfma16(vf[d], pl[t], oacc[d][t]);
      }
      __builtin_amdgcn_sched_barrier(0);
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

// ------------------------------------------------------------------------------------------
// The staged attention with the K and V^T blocks copied from memory straight into LDS (no register pass,
// no LDS stores from registers - those cost bank conflicts whatever the layout - and no registers held
// for data in flight).  A 64-key block is NF one-KiB operand fragments (lane l's 16 bytes at byte 16 l);
// one copy instruction of a wave fills one fragment, each lane fetching the 16 bytes its slot holds: for
// a K fragment (half, tile tt, k-step kk) row 8(c/4) + c%4 + 4tt of the half, bytes 64 kk + 16 g ..,
// for a V^T fragment (half, channel tile d) channel 16 d + c, keys 8g .. 8g+7 of the half (c = l%16,
// g = l/16).  NB buffers form a ring with NB-1 blocks in flight; the only wait on memory is "the block
// about to be multiplied has landed", once per block, before the barrier that also frees the oldest
// buffer.  Needs blocks that never straddle a page (page size a multiple of 64) or the packed scratch.
// The page ids of the sequence are copied into LDS once; rows of a block past the sequence end are read
// as they lie in the page (or workspace) and the V^T columns of such keys are zeroed in LDS before use,
// as are those of a block whose page id is not addressable.
#define DL_VMCNT(n) (((n) & 15) | (((n) >> 4) << 14) | 0x0F70)
template <int DH, int NW, bool PAGED>
__global__ __launch_bounds__(NW * 64) void k_attn_dl(const AttnArgs a) {
  constexpr int KK = DH / 32, DT = DH / 16, QT = 2;
  constexpr int NB = NW >= 8 ? 3 : 2;
  constexpr int NKF = 4 * KK, NVF = 2 * DT, NF = NKF + NVF, FPW = NF / NW;
  static_assert(NF % NW == 0 && NKF % FPW == 0, "a wave's i-th fragment is K for all of a wave or V^T for all");
  constexpr int BLK = NF * 1024, nthr = NW * 64;
  extern __shared__ __attribute__((aligned(1024))) unsigned char dl_smem[];
  int32_t* s_pg = (int32_t*)(dl_smem + NB * BLK);
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
  if (PAGED && a.q_valid && a.q_valid[b] < 0) return;        // the sequence is not part of this call
  const KVView& kv = a.kv;
  const int sh = a.pt_shift, pt = 1 << sh;
  const bf16_t* kslab = (const bf16_t*)kv.k;
  const bf16_t* vslab = (const bf16_t*)kv.v;
  const int64_t pcol = PAGED ? 0 : kv.cu_pad[b];
  bool bad = false;
  const int nkb = (kv_len + 63) >> 6;

  int np = 0;
  if constexpr (PAGED) {
    np = (kv_len + pt - 1) >> sh;
    np = np < a.pg_cap ? np : a.pg_cap;
    np = np < kv.max_pages ? np : kv.max_pages;
    const int32_t* table = kv.table + (int64_t)b * kv.max_pages;
    for (int i = tid; i < np; i += nthr) s_pg[i] = table[i];
  }

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
  __syncthreads();                                            // page ids are in LDS (and the q loads have landed)

  // this lane's source offsets (elements from the block's K or V^T base) for the wave's FPW fragments
  int foff[FPW];
#pragma unroll
  for (int i = 0; i < FPW; ++i) {
    const int f = w * FPW + i;
    if (f < NKF) {
      const int half = f / (2 * KK), tt = (f / KK) & 1, kk = f % KK;
      foff[i] = (half * 32 + 8 * (c >> 2) + (c & 3) + 4 * tt) * DH + (kk * 4 + g) * 8;
    } else {
      const int fv = f - NKF, half = fv / DT, d = fv % DT;
      foff[i] = (d * 16 + c) * (PAGED ? pt : kv.tpad) + half * 32 + g * 8;
    }
  }
  const bool wave_k = w * FPW < NKF;
  uint32_t badbuf = 0;                                        // buffers whose block came from a page id out of range
  auto page_of = [&](int kb64) -> int {
    if constexpr (!PAGED) return 0;
    const int pi = (kb64 << 6) >> sh;
    return pi < np ? s_pg[pi] : -1;
  };
  auto issue = [&](int kb64, int buf, int page_v) {
    const int k0 = kb64 << 6;
    int64_t kb, vb;
    if constexpr (PAGED) {
      const int page = __builtin_amdgcn_readfirstlane(page_v);
      const bool ok = (uint32_t)page < (uint32_t)kv.n_pages;
      bad |= !ok;
      badbuf = ok ? (badbuf & ~(1u << buf)) : (badbuf | (1u << buf));
      const int64_t rows = (((int64_t)(ok ? page : 0) * kv.n_kv_heads + kvh) << sh);
      kb = (rows + (k0 & (pt - 1))) * DH;
      vb = rows * DH + (k0 & (pt - 1));
    } else {
      kb = ((int64_t)kvh * kv.tpad + pcol + k0) * DH;
      vb = (int64_t)kvh * DH * kv.tpad + pcol + k0;
    }
    const bf16_t* src = wave_k ? kslab + kb : vslab + vb;
    unsigned char* dst = dl_smem + buf * BLK + w * FPW * 1024;
#pragma unroll
    for (int i = 0; i < FPW; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + foff[i]),
                                       (__attribute__((address_space(3))) void*)(dst + i * 1024), 16, 0, 0);
  };

  f32x4 oacc[DT][QT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int t = 0; t < QT; ++t) oacc[d][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) { m_run[t] = -DEV_INF; l_run[t] = 0.f; }

  // One 64-key block; the instruction order lets one wave's LDS reads, matrix and vector work overlap
  // (the waves of a workgroup leave the barrier in the same phase): all K fragments are requested first,
  // the scores of both halves issued back to back, each half's V^T fragments requested before its
  // softmax (no LDS traffic: its reductions are row swaps), which runs while the matrix pipe still works.
  auto compute = [&](int buf, int kb64) {
    const int k0 = kb64 << 6;
    const u32x4* fk = (const u32x4*)(dl_smem + buf * BLK) + lane;
    const u32x4* fv = fk + NKF * 64;
    u32x4 kf[2][2][KK];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[half][tt][kk] = fk[((half * 2 + tt) * KK + kk) * 64];
    __builtin_amdgcn_sched_barrier(0);
    f32x4 s[2][2][QT];
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
        for (int t = 0; t < QT; ++t) s[half][tt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
          for (int t = 0; t < QT; ++t) s[half][tt][t] = mfma16(kf[half][tt][kk], qf[t][kk], s[half][tt][t]);
      }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      u32x4 vf[DT];
#pragma unroll
      for (int d = 0; d < DT; ++d) vf[d] = fv[(half * DT + d) * 64];
      __builtin_amdgcn_sched_barrier(0);
      u32x4 pf[QT], pl[QT];
      attn_softmax_block<DT, QT>(s[half], k0 + half * 32, kv_len, g, a.scale_log2, m_run, l_run, oacc, pf, pl);
#pragma unroll
      for (int d = 0; d < DT; ++d) {
#pragma unroll
        for (int t = 0; t < QT; ++t) oacc[d][t] = mfma16(vf[d], pf[t], oacc[d][t]);
#pragma unroll
        for (int t = 0; t < QT; ++t) oacc[d][t] = mfma16(vf[d], pl[t], oacc[d][t]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  if (unit < nkb) {          // (a unit without keys still writes its empty partial below)
    const int last = unit + ((nkb - 1 - unit) / a.n_units) * a.n_units;
    auto clampb = [&](int kb) { return kb <= last ? kb : last; };
    // the ring's first NB-1 blocks (past the end: repeats of the last block into buffers nobody reads)
#pragma unroll
    for (int j = 0; j < NB - 1; ++j) {
      const int kb = clampb(unit + j * a.n_units);
      issue(kb, j, page_of(kb));
    }
    int pg_next = page_of(clampb(unit + (NB - 1) * a.n_units));
    int buf = 0;
    for (int kb = unit; kb < nkb; kb += a.n_units) {
      // (the count is exact only while the loop issues no other vector memory instruction: no spills to scratch,
      // which the build's resource report shows)
      __builtin_amdgcn_s_waitcnt(DL_VMCNT((NB - 2) * FPW));   // this wave's copies of block kb have landed
      __builtin_amdgcn_s_barrier();                            // everybody's have; the previous block's buffer is free
      const int nbuf = buf == 0 ? NB - 1 : buf - 1;            // (buf + NB - 1) % NB: the buffer of the block before
      const int kn = clampb(kb + (NB - 1) * a.n_units);
      issue(kn, nbuf, pg_next);
      pg_next = page_of(clampb(kb + NB * a.n_units));
      if ((kb << 6) + 64 > kv_len || ((badbuf >> buf) & 1u)) {
        // zero the V^T columns of keys past the sequence end (all keys of a block without a page)
        const bool nopage = (badbuf >> buf) & 1u;
        u32x4* vb = (u32x4*)(dl_smem + buf * BLK + NKF * 1024);
        for (int q = tid; q < NVF * 64; q += nthr) {
          const int half = (q >> 6) / DT, gg = (q & 63) >> 4;
          const int valid = nopage ? 0 : kv_len - ((kb << 6) + half * 32 + gg * 8);
          if (valid < 8) {
            u32x4 v = vb[q];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              uint32_t x = v[e];
              x = valid > 2 * e + 1 ? x : (x & 0x0000ffffu);
              x = valid > 2 * e ? x : 0u;
              v[e] = x;
            }
            vb[q] = v;
          }
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
      }
      if (active) compute(buf, kb);
      buf = buf + 1 == NB ? 0 : buf + 1;
    }
    __builtin_amdgcn_s_waitcnt(DL_VMCNT(0));   // the trailing repeats must not outlive the workgroup
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
constexpr int DL_LDS_MAX = 128 * 1024;          // ring of k_attn_dl plus its copy of a sequence's page ids
hipError_t init_attn_kernels() {
  if (attn_merge_ready) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)k_attn_step<128, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_attn_step<64, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
#define DL_ATTR(DHV, NWV, PG)                                                                                     \
  if (e == hipSuccess)                                                                                            \
    e = hipFuncSetAttribute((const void*)k_attn_dl<DHV, NWV, PG>, hipFuncAttributeMaxDynamicSharedMemorySize, DL_LDS_MAX)
  DL_ATTR(128, 8, true); DL_ATTR(128, 8, false); DL_ATTR(128, 4, true); DL_ATTR(128, 4, false);
  DL_ATTR(64, 8, true); DL_ATTR(64, 8, false); DL_ATTR(64, 4, true); DL_ATTR(64, 4, false);
#undef DL_ATTR
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
  int pt_shift = 0;
  if (g.Q > 0) {
    pt_shift = -1;
    for (int sft = 3; sft < 31; ++sft) if (f.page_tokens == (1 << sft)) pt_shift = sft;
  }
  const bool staged = n_rg >= 4 && pt_shift >= 0;   // K/V staged in LDS, up to 8 row groups per workgroup
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
    // blocks inside one page (or the packed scratch): straight-to-LDS copies, if the ring and the sequence's
    // page ids fit; otherwise the loader that goes through registers
    a.pg_cap = paged ? (g.max_kv + f.page_tokens - 1) / f.page_tokens : 0;
    const size_t ring = (size_t)(n_rg_wg <= 4 ? 2 : 3) * (size_t)(f.head_dim / 4) * 1024;   // NB buffers of head_dim/4 one-KiB fragments
    const size_t dl_lds = ring + (size_t)a.pg_cap * sizeof(int32_t);
    const bool direct = fast && attn_merge_ready && dl_lds <= (size_t)DL_LDS_MAX;
#define ATTN_LDS(DHV, NWV)                                                                                 \
  do {                                                                                                     \
    if (direct && paged) k_attn_dl<DHV, NWV, true><<<grid, NWV * 64, dl_lds, s>>>(a);                      \
    else if (direct) k_attn_dl<DHV, NWV, false><<<grid, NWV * 64, dl_lds, s>>>(a);                         \
    else if (!paged) k_attn_lds<DHV, NWV, false, true><<<grid, NWV * 64, 0, s>>>(a);                       \
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
