// Per-step passes over the decompression matrices (bases) in 16-bit storage: bandwidth-bound
// matrix-vector products that read every basis byte exactly once, whole rows at a time.
//
//   basis_rows<DOT, FOLD>   one pass over Bm [r, HD] of every sequence, each wave streaming
//                           whole rows (HD contiguous elements, 128-bit loads, several rows
//                           in flight) and producing, per row j,
//       DOT :  c[j]     = Bm[j, :] . x                 the appended token's coefficient
//                                                      (paper Sec. 3.1 projection, one row)
//       FOLD:  q'[h, j] = scale * Bm[j, head h] . q_h  the query folded through the key basis
//                                                      (Alg. 1 scores by associativity)
//                           With both, the append of a key row and the fold of the query
//                           share one pass over B_k.
//   merge_expand            combine the token splits of attn_partial and expand through B_v:
//                           out[h, :] = (sum_s w_s U_s[h, :] / sum_s w_s l_s) . Bv[:, head h]
//                           (Alg. 1 output by associativity).  A workgroup owns two heads
//                           (512-byte row segments) and keeps eight rows in flight per thread.
// Products of two 16-bit values are exact in fp32; sums are fp32 (v_dot2c_f32_*).
#include "ap_common.hpp"
#include "lane_ops.hpp"

namespace ap {
namespace {

struct RowsParams {
  const uint16_t* Bm;     // [B][r][HD] (bstride elements between sequences, 0 = shared)
  int64_t bstride;
  const uint16_t* x;      // DOT:  [B][HD] the token row to project
  const uint16_t* q;      // FOLD: [B][H][d] (= [B][HD])
  uint16_t* C;            // DOT:  [B][T_cap][r], row `row0` written
  uint16_t* Qp;           // FOLD: [B][2][Hp][r] hi / lo parts of the folded query
  int H, Hp, d, HD, r, row0, T_cap;
  int rpw;                // consecutive rows per wave (a workgroup owns 4 * rpw rows)
  float scale;
  // PAIR: a second DOT job of the same shape in the same launch (blockIdx.z = 1), e.g. the
  // value row of a step appended next to the key row
  const uint16_t* Bm2;
  const uint16_t* x2;
  uint16_t* C2;
};

template <class Tag>
__device__ __forceinline__ void split_hi_lo(float x, uint16_t& hi, uint16_t& lo) {
  hi = f32_to_bits(x, Tag{});
  lo = f32_to_bits(x - bits_to_f32(hi, Tag{}), Tag{});
}

// grid (ceil(r / (4 rpw)), B), 256 threads.  KPC = 512-element passes that cover the hidden
// axis; a wave walks its rows through a ring of NBUF row buffers in registers, so NBUF - 1
// rows (HD * 2 bytes each) are in flight while one is reduced.
// LPH = d / 8 lanes share a head (FOLD; 1 when the kernel does not fold).
// PAIR: grid.z = 2; the workgroups of z = 1 run the second job (DOT only) on Bm2, x2, C2.
template <class Tag, int KPC, int NBUF, bool DOT, bool FOLD, int LPH, bool PAIR = false>
__global__ void __launch_bounds__(256) basis_rows(const RowsParams p) {
  extern __shared__ __attribute__((aligned(16))) float qtile[];   // FOLD: [Hp][4 rpw + 1]
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rpw = p.rpw, rows_wg = 4 * rpw, pitch = rows_wg + 1;
  const int b = blockIdx.y, j0 = blockIdx.x * rows_wg;
  const int HD = p.HD, r = p.r;
  const bool second = PAIR && blockIdx.z == 1;
  const bool fold = FOLD && !second;
  const uint16_t* Bb = (second ? p.Bm2 : p.Bm) + (size_t)b * p.bstride;
  const uint16_t* xv = second ? p.x2 : p.x;
  uint16_t* Cb = second ? p.C2 : p.C;
  u32x4_t buf[NBUF][KPC];
  // passes beyond the hidden axis re-read the lane's first chunk (their vector slices are
  // zero), so the loads carry no branches and issue back to back
  int eoff[KPC];
#pragma unroll
  for (int pp = 0; pp < KPC; ++pp)
    eoff[pp] = (pp * 512 + lane * 8) < HD ? pp * 512 + lane * 8 : (lane * 8 < HD ? lane * 8 : 0);
  auto load_row = [&](u32x4_t (&dst)[KPC], int i) {         // row i of this wave
    int j = j0 + w * rpw + i;
    j = j < r ? j : r - 1;                                  // rows past the end: harmless repeats
    const uint16_t* row = Bb + (size_t)j * HD;
#pragma unroll
    for (int pp = 0; pp < KPC; ++pp) {
      // wide rows (read once per launch) are streamed with the non-temporal hint, which pays only
      // with a shallow ring: at HD = 5120 one row in flight per wave and the hint 77 us, two rows
      // in flight 80 us without and 87 us with it
      if constexpr (KPC == 10) dst[pp] = __builtin_nontemporal_load((const u32x4_t*)(row + eoff[pp]));
      else dst[pp] = *(const u32x4_t*)(row + eoff[pp]);
    }
  };
  // this lane's slices of the vectors: elements 512 pp + 8 lane .. +7 of the hidden axis.
  // They are requested BEFORE the first rows, so that a row's arrival implies theirs and no
  // wait on them ever drains the row ring.
  u32x4_t xs[DOT ? KPC : 1], qs[FOLD ? KPC : 1];
#pragma unroll
  for (int pp = 0; pp < KPC; ++pp) {
    const int e0 = pp * 512 + lane * 8;
    const u32x4_t z = {0, 0, 0, 0};
    if (DOT) xs[pp] = e0 < HD ? *(const u32x4_t*)(xv + (size_t)b * HD + e0) : z;
    if (FOLD) qs[pp] = e0 < HD && fold ? *(const u32x4_t*)(p.q + (size_t)b * HD + e0) : z;
  }
  const int last = rpw - 1;
#pragma unroll
  for (int u = 0; u + 1 < NBUF; ++u) load_row(buf[u], u < last ? u : last);
  if (fold) {
    for (int i = tid; i < p.Hp * pitch; i += 256) qtile[i] = 0.f;   // padded heads stay 0
    __syncthreads();
  }
  constexpr int dshift = FOLD ? 31 - __builtin_clz((unsigned)(LPH * 8)) : 0;   // log2(d)

  auto reduce_row = [&](const u32x4_t (&row)[KPC], int i) {
    const int jl = w * rpw + i;
    const bool live = i < rpw && j0 + jl < r;
    if (DOT) {
      float acc = 0.f;
#pragma unroll
      for (int pp = 0; pp < KPC; ++pp) acc = dot8<Tag>(row[pp], xs[pp], acc);
      acc = wave_sum(acc);
      if (lane == 0 && live)
        Cb[((size_t)b * p.T_cap + p.row0) * r + j0 + jl] = f32_to_bits(acc, Tag{});
    }
    if (fold) {
#pragma unroll
      for (int pp = 0; pp < KPC; ++pp) {
        float part = dot8<Tag>(row[pp], qs[pp], 0.f);
        part = group_sum<LPH>(part);
        const int e0 = pp * 512 + lane * 8;
        if ((lane & (LPH - 1)) == 0 && e0 < HD && live)
          qtile[(e0 >> dshift) * pitch + jl] = part * p.scale;
      }
    }
  };
  // The ring advances without branches: every slot of the unrolled body requests a row and
  // reduces one (past the wave's last row the request repeats that row, a cache hit, and the
  // reduction's result is dropped), so the compiler's wait counts stay exact.
  const int rpw_pad = (rpw + NBUF - 1) / NBUF * NBUF;
  for (int i = 0; i < rpw_pad; i += NBUF) {
#pragma unroll
    for (int u = 0; u < NBUF; ++u) {
      const int nx = i + u + NBUF - 1;
      load_row(buf[(u + NBUF - 1) % NBUF], nx < last ? nx : last);
      reduce_row(buf[u], i + u);
    }
  }
  if (fold) {
    __syncthreads();
    // consecutive rank positions of one head leave as one contiguous segment per part
    for (int i = tid; i < p.Hp * rows_wg; i += 256) {
      const int h = i / rows_wg, jl = i - h * rows_wg;
      if (j0 + jl < r) {
        uint16_t hi, lo;
        split_hi_lo<Tag>(qtile[h * pitch + jl], hi, lo);
        p.Qp[(((size_t)b * 2 + 0) * p.Hp + h) * r + j0 + jl] = hi;
        p.Qp[(((size_t)b * 2 + 1) * p.Hp + h) * r + j0 + jl] = lo;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// fold_heads: the fold for grouped queries, q'[h, j] = scale * Bk[j, slice of key/value head
// h / G] . q_h.  A workgroup owns one key/value head and 64 basis rows; groups of LPH = d / 8
// lanes take one row each (four rows in flight per group) and dot it with the queries of all
// G heads that share the slice, so every basis byte is loaded once.
//   grid (H_kv * ceil(G / 8), ceil(r / 64), B), 256 threads; the workgroups of key/value
//   head 0 also write the padding heads H .. Hp-1 as zeros.
// ------------------------------------------------------------------------------------------
template <class Tag, int LPH>
__global__ void __launch_bounds__(256)
fold_heads(const uint16_t* __restrict__ Bk, int64_t bstride, const uint16_t* __restrict__ q,
           uint16_t* __restrict__ Qp, int H, int G, int Hp, int r, float scale) {
  constexpr int d = LPH * 8;
  constexpr int NG = 256 / LPH;                 // rows per pass of the workgroup
  const int nsub = (G + 7) >> 3;                // query heads are taken eight at a time
  const int kvh = blockIdx.x / nsub, sub = blockIdx.x - kvh * nsub;
  const int b = blockIdx.z, tid = threadIdx.x;
  const int jb = blockIdx.y * 64;
  int jend = jb + 64;
  jend = jend < r ? jend : r;
  if (blockIdx.x == 0) {
    for (int i = tid; i < (Hp - H) * (jend - jb); i += 256) {
      const int h = H + i / (jend - jb), j = jb + i % (jend - jb);
      Qp[(((size_t)b * 2 + 0) * Hp + h) * r + j] = 0;
      Qp[(((size_t)b * 2 + 1) * Hp + h) * r + j] = 0;
    }
  }
  const int g = tid / LPH, li = tid % LPH;
  const size_t HD = (size_t)(H / G) * d;
  const int h0 = kvh * G + sub * 8;             // first query head of this workgroup
  int nq = G - sub * 8;
  nq = nq < 8 ? nq : 8;
  u32x4_t qv[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int hk = k < nq ? h0 + k : h0;        // unused slots repeat the first head
    qv[k] = *(const u32x4_t*)(q + ((size_t)b * H + hk) * d + li * 8);
  }
  const uint16_t* col = Bk + (size_t)b * bstride + (size_t)kvh * d + li * 8;
  for (int j0 = jb; j0 < jend; j0 += NG * 4) {
    u32x4_t rowv[4];
    int j[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      j[u] = j0 + u * NG + g;
      const int jc = j[u] < jend ? j[u] : jend - 1;          // in-bounds repeat, result dropped
      rowv[u] = *(const u32x4_t*)(col + (size_t)jc * HD);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (k < nq) {                                         // wave-uniform
          const float v = group_sum<LPH>(dot8<Tag>(rowv[u], qv[k], 0.f)) * scale;
          if (li == 0 && j[u] < jend) {
            uint16_t hi, lo;
            split_hi_lo<Tag>(v, hi, lo);
            Qp[(((size_t)b * 2 + 0) * Hp + h0 + k) * r + j[u]] = hi;
            Qp[(((size_t)b * 2 + 1) * Hp + h0 + k) * r + j[u]] = lo;
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// merge_expand: grid (ceil(H / 2), B), 256 threads.
// ------------------------------------------------------------------------------------------
template <class Tag, bool OUT_F32, int kS>
__global__ void __launch_bounds__(256)
merge_expand(const float* __restrict__ part_ml, const float* __restrict__ part_U,
             const uint16_t* __restrict__ Bv, int64_t bstride, void* __restrict__ out,
             float* __restrict__ lse, int H, int G, int d, int r, int nsplit) {
  extern __shared__ __attribute__((aligned(16))) char smem_me[];
  float* ustar = (float*)smem_me;          // [2][r]
  float* red = ustar + 2 * r;              // [rows][2 d]
  const int h0 = blockIdx.x * 2, b = blockIdx.y, tid = threadIdx.x;
  const int nh = H - h0 < 2 ? H - h0 : 2;  // heads of this workgroup
  // ---- merged, normalised coefficient sums of the two heads.  At most kS (8 or 16) splits
  //      arrive here (more are merged beforehand); every load of a thread is issued before the
  //      first is used, so the prologue costs two memory round trips, not one per split.
  for (int i = tid; i < nh * r; i += 256) {
    const int hh = i >= r ? 1 : 0, j = i - hh * r;
    const size_t pb = (size_t)b * nsplit * H + h0 + hh;    // + s*H
    float ms[kS], ls[kS], us_[kS];
#pragma unroll
    for (int s = 0; s < kS; ++s) {
      const size_t ps = pb + (size_t)(s < nsplit ? s : 0) * H;
      ms[s] = part_ml[ps * 2];
      ls[s] = part_ml[ps * 2 + 1];
      us_[s] = part_U[ps * r + j];
    }
    float mstar = -INFINITY;
#pragma unroll
    for (int s = 0; s < kS; ++s) if (s < nsplit) mstar = fmaxf(mstar, ms[s]);
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int s = 0; s < kS; ++s) {
      if (s < nsplit) {
        const float ws = fast_exp2(ms[s] - mstar);
        L = fmaf(ls[s], ws, L);
        acc = fmaf(ws, us_[s], acc);
      }
    }
    ustar[hh * r + j] = acc / L;
    if (j == 0 && lse) lse[(size_t)b * H + h0 + hh] = (mstar + log2f(L)) * kLn2;
  }
  __syncthreads();
  // ---- expansion: thread (rg, cc) owns 8 columns of the 2d-wide slice and rows rg, rg+rows, ..
  const int tpr = (2 * d) >> 3;            // threads per row segment: 8 .. 64
  const int rows = 256 / tpr;
  const int rg = tid / tpr, cc = tid - rg * tpr;
  const bool live = cc * 8 < nh * d;       // an odd head count leaves the upper half idle
  const float* us = ustar + (cc * 8 >= d ? r : 0);
  // grouped queries: G consecutive query heads read the same d-wide slice of the basis rows
  const size_t HD = (size_t)(H / G) * d;
  const int hsel = cc * 8 >= d ? 1 : 0;
  const uint16_t* Bb = Bv + (size_t)b * bstride + (size_t)((h0 + hsel) / G) * d + (cc * 8 - hsel * d);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (live) {
    int j = rg;
    for (; j + 7 * rows < r; j += 8 * rows) {              // eight rows in flight
      u32x4_t wv[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) wv[k] = *(const u32x4_t*)(Bb + (size_t)(j + k * rows) * HD);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float u = us[j + k * rows];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[2 * e] = fmaf(u, lo_to_f32(wv[k][e], Tag{}), acc[2 * e]);
          acc[2 * e + 1] = fmaf(u, hi_to_f32(wv[k][e], Tag{}), acc[2 * e + 1]);
        }
      }
    }
    for (; j + 3 * rows < r; j += 4 * rows) {              // four rows in flight
      u32x4_t wv[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) wv[k] = *(const u32x4_t*)(Bb + (size_t)(j + k * rows) * HD);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float u = us[j + k * rows];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[2 * e] = fmaf(u, lo_to_f32(wv[k][e], Tag{}), acc[2 * e]);
          acc[2 * e + 1] = fmaf(u, hi_to_f32(wv[k][e], Tag{}), acc[2 * e + 1]);
        }
      }
    }
    for (; j < r; j += rows) {
      const u32x4_t wv = *(const u32x4_t*)(Bb + (size_t)j * HD);
      const float u = us[j];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] = fmaf(u, lo_to_f32(wv[e], Tag{}), acc[2 * e]);
        acc[2 * e + 1] = fmaf(u, hi_to_f32(wv[e], Tag{}), acc[2 * e + 1]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rg * 2 * d + cc * 8 + e] = acc[e];
  __syncthreads();
  for (int i = tid; i < nh * d; i += 256) {
    float sum = 0.f;
    for (int k = 0; k < rows; ++k) sum += red[k * 2 * d + i];
    const size_t o = ((size_t)b * H + h0) * d + i;
    if (OUT_F32) ((float*)out)[o] = sum;
    else ((uint16_t*)out)[o] = f32_to_bits(sum, Tag{});
  }
}


// ------------------------------------------------------------------------------------------
// expand_append: the expansion through B_v and the append of the new token's value row in ONE
// pass over B_v (a fused decode step).  attn_partial has scored all T tokens but summed the
// value coefficients of the T-1 older ones only, exporting the newest token's softmax weight;
// that token's weighted coefficient sum is its own coefficient row c_v[j] = B_v[j, :] . v_new,
// which a whole-row pass produces row by row.  So for basis row j
//     U*[h, j]  = A[h, j] + beta[h] * c_v[j]
//     out[h, :] += U*[h, j] * B_v[j, head h]
// with A the merged, normalised partial sums of the older tokens and beta[h] the new token's
// softmax weight.  A workgroup owns a block of rows; its per-column sums go to a partial buffer
// that reduce_out adds up in a fixed order (deterministic).
//   grid (ceil(r / rpw), B), 128 threads; dynamic LDS: A [H][rpw + 1], statistics.
// ------------------------------------------------------------------------------------------
struct ExpandParams {
  const uint16_t* Bv;
  int64_t bstride;
  const uint16_t* v_new;    // [B][HD]
  uint16_t* Cv;             // [B][T_cap][r]: row T-1 is written
  const float* part_ml;     // [B][S][H][2] (reference exponent, sum) over all T tokens
  const float* part_U;      // [B][S][H][r] over tokens 0 .. T-2
  const float* pnew;        // [B][H] weight of token T-1 relative to the reference of the split that holds it
  const int* pnew_split;    // [B] that split, or null: the last one
  const int32_t* rank_v;    // [B][T] per-token value ranks, or null: the new token counts at rank r
  float* pout;              // [B][nob][HD] per-row-block column sums
  float* lse;               // [B][H] or null
  int H, d, HD, r, T, T_cap, nsplit, rpw, nob;
};

template <class Tag, int KPC, int NBUF>
__global__ void __launch_bounds__(128) expand_append(const ExpandParams p) {
  // Two waves share the workgroup's rows, each owning KPC / 2 of the 512-element passes over
  // the hidden axis (so the column sums fit in registers); the two halves of a row's dot
  // product meet in LDS once per row.
  constexpr int KH = KPC / 2;
  extern __shared__ __attribute__((aligned(16))) float lds_ea[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int half = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rpw = p.rpw, pitch = rpw + 1;
  const int b = blockIdx.y, j0 = blockIdx.x * rpw;
  const int H = p.H, HD = p.HD, r = p.r, S = p.nsplit;
  float* Atile = lds_ea;                       // [H][pitch]
  float* mstar = Atile + H * pitch;            // [H]
  float* invL = mstar + H;                     // [H]
  float* beta = invL + H;                      // [H]
  float* dotx = beta + H;                      // [2][2] half dot products, double-buffered
  float* wsp = dotx + 4;                       // [S][H] split weights (when they fit)
  const bool wsp_fits = S * H <= 4096;
  const uint16_t* Bb = p.Bv + (size_t)b * p.bstride;

  // ---- row ring: requests go out first (see basis_rows)
  u32x4_t buf[NBUF][KH];
  int eoff[KH];
  bool inside[KH];
#pragma unroll
  for (int pp = 0; pp < KH; ++pp) {
    const int e0 = (half * KH + pp) * 512 + lane * 8;
    inside[pp] = e0 < HD;
    eoff[pp] = inside[pp] ? e0 : (lane * 8 < HD ? lane * 8 : 0);
  }
  auto load_row = [&](u32x4_t (&dst)[KH], int i) {
    int j = j0 + i;
    j = j < r ? j : r - 1;
    const uint16_t* row = Bb + (size_t)j * HD;
#pragma unroll
    // (a basis row is read once per launch: non-temporal, measured 92.2 -> 88.3 us; the same hint
    // costs basis_rows 7 us and is not used there)
    for (int pp = 0; pp < KH; ++pp) dst[pp] = __builtin_nontemporal_load((const u32x4_t*)(row + eoff[pp]));
  };
  u32x4_t vs[KH];
#pragma unroll
  for (int pp = 0; pp < KH; ++pp) {
    const u32x4_t z = {0, 0, 0, 0};
    vs[pp] = inside[pp] ? *(const u32x4_t*)(p.v_new + (size_t)b * HD + eoff[pp]) : z;
  }
  const int last = rpw - 1;
#pragma unroll
  for (int u = 0; u + 1 < NBUF; ++u) load_row(buf[u], u < last ? u : last);

  // ---- merged softmax statistics: one thread per head
  if (tid < H) {
    const int h = tid;
    const size_t pb = (size_t)b * S * H + h;
    // the splits' (reference exponent, sum) pairs, eight loads in flight at a time
    float m = -INFINITY;
    for (int s0 = 0; s0 < S; s0 += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = s0 + u < S ? p.part_ml[(pb + (size_t)(s0 + u) * H) * 2] : -INFINITY;
#pragma unroll
      for (int u = 0; u < 8; ++u) m = fmaxf(m, v[u]);
    }
    float L = 0.f, wlast = 0.f;
    const int snew = p.pnew_split ? p.pnew_split[b] : S - 1;
    for (int s0 = 0; s0 < S; s0 += 8) {
      float v[8], lv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool on = s0 + u < S;
        v[u] = on ? p.part_ml[(pb + (size_t)(s0 + u) * H) * 2] : -INFINITY;
        lv[u] = on ? p.part_ml[(pb + (size_t)(s0 + u) * H) * 2 + 1] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (s0 + u < S) {
          const float ws = fast_exp2(v[u] - m);
          L += lv[u] * ws;
          if (wsp_fits) wsp[(s0 + u) * H + h] = ws;
          if (s0 + u == snew) wlast = ws;
        }
      }
    }
    mstar[h] = m;
    invL[h] = 1.0f / L;
    beta[h] = wlast * p.pnew[(size_t)b * H + h] / L;
    if (p.lse && blockIdx.x == 0) p.lse[(size_t)b * H + h] = (m + log2f(L)) * kLn2;
  }
  __syncthreads();
  // ---- A[h][jl] = sum_s 2^(m_s - m*) U_s[h, j0 + jl] / L
  if (wsp_fits) {
    // four (head, row) pairs and four splits at a time: sixteen loads in flight per thread, so
    // the whole tile takes a few round trips to memory (the row ring stands still meanwhile)
    const int n = H * rpw;
    for (int i0 = tid; i0 < n; i0 += 4 * 128) {
      int hh[4], jj[4];
      bool ok[4];
      size_t base[4];
      float acc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + 128 * u;
        const int h = i < n ? i / rpw : 0, jl = i < n ? i - h * rpw : 0;
        hh[u] = h;
        jj[u] = jl;
        ok[u] = i < n && j0 + jl < r;
        base[u] = ((size_t)b * S * H + h) * r + (ok[u] ? j0 + jl : 0);
        acc[u] = 0.f;
      }
      for (int s0 = 0; s0 < S; s0 += 4) {
        float uv[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int k = 0; k < 4; ++k)
            uv[u][k] = s0 + k < S ? p.part_U[base[u] + (size_t)(s0 + k) * H * r] : 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (s0 + k < S) acc[u] = fmaf(wsp[(s0 + k) * H + hh[u]], uv[u][k], acc[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (i0 + 128 * u < n) Atile[hh[u] * pitch + jj[u]] = ok[u] ? acc[u] * invL[hh[u]] : 0.f;
    }
  } else {
    for (int i = tid; i < H * rpw; i += 128) {
      const int h = i / rpw, jl = i - h * rpw;
      float acc = 0.f;
      if (j0 + jl < r) {
        const size_t pb = (size_t)b * S * H + h;
        const float m = mstar[h];
        for (int s = 0; s < S; ++s)
          acc = fmaf(fast_exp2(p.part_ml[(pb + (size_t)s * H) * 2] - m),
                     p.part_U[(pb + (size_t)s * H) * r + j0 + jl], acc);
        acc *= invL[h];
      }
      Atile[h * pitch + jl] = acc;
    }
  }
  __syncthreads();

  // the new token's own value rank limits the rows in which its coefficient counts
  int rvn = r;
  if (p.rank_v) {
    rvn = p.rank_v[(size_t)b * p.T + p.T - 1];
    rvn = rvn < 0 ? 0 : (rvn < r ? rvn : r);
  }
  const int dshift = 31 - __builtin_clz((unsigned)p.d);
  float bt[KH];
  int arow[KH];                                // A row (head) of this lane's chunk in every pass
#pragma unroll
  for (int pp = 0; pp < KH; ++pp) {
    const int h = inside[pp] ? eoff[pp] >> dshift : 0;
    bt[pp] = inside[pp] ? beta[h] : 0.f;
    arow[pp] = h * pitch;
  }
  float o[KH][8];
#pragma unroll
  for (int pp = 0; pp < KH; ++pp)
#pragma unroll
    for (int e = 0; e < 8; ++e) o[pp][e] = 0.f;

  auto use_row = [&](const u32x4_t (&row)[KH], int i) {
    const bool live = i < rpw && j0 + i < r;
    float acc = 0.f;
#pragma unroll
    for (int pp = 0; pp < KH; ++pp) acc = dot8<Tag>(row[pp], vs[pp], acc);
    acc = wave_sum(acc);
    float* slot = dotx + (i & 1) * 2;
    if (lane == 0) slot[half] = acc;
    // both waves run the same number of rows.  Only LDS traffic has to be ordered here: a full
    // __syncthreads() would also wait for the row loads in flight and drain the ring.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const float c = slot[0] + slot[1];
    const uint16_t cbits = f32_to_bits(c, Tag{});
    if (lane == 0 && half == 0 && live) p.Cv[((size_t)b * p.T_cap + p.T - 1) * r + j0 + i] = cbits;
    const float cr = live && j0 + i < rvn ? bits_to_f32(cbits, Tag{}) : 0.f;   // the stored (rounded) coefficient
    const int jc = live ? i : 0;
#pragma unroll
    for (int pp = 0; pp < KH; ++pp) {
      const float wgt = live ? fmaf(bt[pp], cr, Atile[arow[pp] + jc]) : 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[pp][2 * e] = fmaf(wgt, lo_to_f32(row[pp][e], Tag{}), o[pp][2 * e]);
        o[pp][2 * e + 1] = fmaf(wgt, hi_to_f32(row[pp][e], Tag{}), o[pp][2 * e + 1]);
      }
    }
  };
  const int rpw_pad = (rpw + NBUF - 1) / NBUF * NBUF;
  for (int i = 0; i < rpw_pad; i += NBUF) {
#pragma unroll
    for (int u = 0; u < NBUF; ++u) {
      const int nx = i + u + NBUF - 1;
      if (NBUF > 1) load_row(buf[(u + NBUF - 1) % NBUF], nx < last ? nx : last);
      else load_row(buf[0], i < last ? i : last);
      use_row(buf[u], i + u);
    }
  }
  // ---- the two waves own disjoint columns: straight to the partial buffer
  float* dst = p.pout + ((size_t)b * p.nob + blockIdx.x) * HD;
#pragma unroll
  for (int pp = 0; pp < KH; ++pp) {
    if (inside[pp]) {
      const f32x4_t v0 = {o[pp][0], o[pp][1], o[pp][2], o[pp][3]};
      const f32x4_t v1 = {o[pp][4], o[pp][5], o[pp][6], o[pp][7]};
      *(f32x4_t*)(dst + eoff[pp]) = v0;
      *(f32x4_t*)(dst + eoff[pp] + 4) = v1;
    }
  }
}

// out[b, c] = sum over row blocks of pout[b][blk][c], in block order.  grid (ceil(HD/1024), B).
template <class Tag, bool OUT_F32>
__global__ void __launch_bounds__(256)
reduce_out(const float* __restrict__ pout, void* __restrict__ out, int HD, int nob) {
  const int b = blockIdx.y, c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= HD) return;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  int k = 0;
  for (; k + 8 <= nob; k += 8) {                         // eight loads in flight, summed in block order
    f32x4_t v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = *(const f32x4_t*)(pout + ((size_t)b * nob + k + u) * HD + c);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  for (; k < nob; ++k) acc += *(const f32x4_t*)(pout + ((size_t)b * nob + k) * HD + c);
  if (OUT_F32) {
    *(f32x4_t*)((float*)out + (size_t)b * HD + c) = acc;
  } else {
    u32x2_t v = {pack2(acc[0], acc[1], Tag{}), pack2(acc[2], acc[3], Tag{})};
    *(u32x2_t*)((uint16_t*)out + (size_t)b * HD + c) = v;
  }
}


// ------------------------------------------------------------------------------------------
// merge_splits: many token splits (small batches) are merged once, in parallel, before the
// expansion: U'[h, j] = sum_s 2^(m_s - m*) U_s[h, j], l' = sum_s 2^(m_s - m*) l_s, m' = m*, written
// as a single split, and the deferred token's weight is rescaled to the merged reference.
//   grid (ceil(r / 64), H, B), 256 threads = 4 groups of splits x 64 columns.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
merge_splits(const float* __restrict__ part_ml, const float* __restrict__ part_U,
             float* __restrict__ out_ml, float* __restrict__ out_U, float* __restrict__ pnew,
             const int* __restrict__ pnew_split, int H, int r, int S) {
  extern __shared__ __attribute__((aligned(16))) float lds_ms[];   // [S] weights, then [4][64]
  __shared__ float red[8];
  const int tid = threadIdx.x, lane = tid & 63, grp = tid >> 6;
  const int h = blockIdx.y, b = blockIdx.z;
  const size_t pb = (size_t)b * S * H + h;                 // + s*H
  float* wgt = lds_ms;
  float* acc4 = lds_ms + S;
  // m* = max_s m_s
  float m = -INFINITY;
  for (int s = tid; s < S; s += 256) m = fmaxf(m, part_ml[(pb + (size_t)s * H) * 2]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if (lane == 0) red[grp] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float L = 0.f;
  for (int s = tid; s < S; s += 256) {
    const float ws = fast_exp2(part_ml[(pb + (size_t)s * H) * 2] - m);
    wgt[s] = ws;
    L += ws * part_ml[(pb + (size_t)s * H) * 2 + 1];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) L += __shfl_xor(L, o);
  if (lane == 0) red[4 + grp] = L;
  __syncthreads();
  L = (red[4] + red[5]) + (red[6] + red[7]);
  const int j = blockIdx.x * 64 + lane;
  float acc = 0.f;
  if (j < r) {
    int s = grp;
    for (; s + 28 < S; s += 32) {                          // eight loads in flight
      float u[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) u[k] = part_U[(pb + (size_t)(s + 4 * k) * H) * r + j];
#pragma unroll
      for (int k = 0; k < 8; ++k) acc = fmaf(wgt[s + 4 * k], u[k], acc);
    }
    for (; s < S; s += 4) acc = fmaf(wgt[s], part_U[(pb + (size_t)s * H) * r + j], acc);
  }
  acc4[grp * 64 + lane] = acc;
  __syncthreads();
  if (grp == 0 && j < r)
    out_U[((size_t)b * H + h) * r + j] = (acc4[lane] + acc4[64 + lane]) + (acc4[128 + lane] + acc4[192 + lane]);
  if (blockIdx.x == 0 && tid == 0) {
    out_ml[((size_t)b * H + h) * 2] = m;
    out_ml[((size_t)b * H + h) * 2 + 1] = L;
    if (pnew) pnew[(size_t)b * H + h] *= wgt[pnew_split ? pnew_split[b] : S - 1];   // its split's weight
  }
}

}  // namespace
int basis_rows_per_wave(int B, int r);
namespace {

template <class Tag, bool DOT, bool FOLD, bool PAIR>
ap_status launch_rows(RowsParams p, int B, hipStream_t stream) {
  const int rpw = basis_rows_per_wave(B, p.r);
  p.rpw = rpw;
  const int rows_wg = 4 * rpw;
  const dim3 grid((p.r + rows_wg - 1) / rows_wg, B, PAIR ? 2 : 1);
  const size_t lds = FOLD ? (size_t)p.Hp * (rows_wg + 1) * 4 : 0;
  const int kpc = (p.HD + 511) / 512;
#define AP_ROWS(K, NB)                                                                        \
  if (kpc <= K) {                                                                             \
    if (!FOLD) hipLaunchKernelGGL((basis_rows<Tag, K, NB, DOT, FOLD, 1, PAIR>), grid, dim3(256), lds, stream, p);            \
    else if (p.d == 128) hipLaunchKernelGGL((basis_rows<Tag, K, NB, DOT, FOLD, FOLD ? 16 : 1, PAIR>), grid, dim3(256), lds, stream, p); \
    else if (p.d == 64) hipLaunchKernelGGL((basis_rows<Tag, K, NB, DOT, FOLD, FOLD ? 8 : 1, PAIR>), grid, dim3(256), lds, stream, p);   \
    else if (p.d == 256) hipLaunchKernelGGL((basis_rows<Tag, K, NB, DOT, FOLD, FOLD ? 32 : 1, PAIR>), grid, dim3(256), lds, stream, p); \
    else hipLaunchKernelGGL((basis_rows<Tag, K, NB, DOT, FOLD, FOLD ? 4 : 1, PAIR>), grid, dim3(256), lds, stream, p);                  \
    return AP_OK;                                                                             \
  }
  AP_ROWS(2, 3) AP_ROWS(4, 3) AP_ROWS(8, 3) AP_ROWS(10, 2)
  AP_ROWS(16, (DOT && FOLD) ? 1 : 2)
#undef AP_ROWS
  set_error("basis pass: H*d=%d exceeds 8192", p.HD);
  return AP_ERR_UNSUPPORTED;
}

}  // namespace

bool basis_rows_applies(int HD, int B) { return HD % 8 == 0 && HD <= 8192 && B <= 65535; }

// Append (x != null) and / or fold (q != null) in one pass over Bm.  With Bm2, x2, C2 (and x)
// given, a second append of the same shape (C2's row row0 = Bm2 . x2) runs in the same launch.
ap_status launch_basis_rows(ap_dtype dt, const void* Bm, int64_t bstride, const void* x,
                            const void* q, void* C, void* Qp, int B, int H, int Hp, int d, int HD,
                            int r, int row0, int T_cap, float scale, hipStream_t stream,
                            const void* Bm2, const void* x2, void* C2) {
  RowsParams p{(const uint16_t*)Bm, bstride, (const uint16_t*)x, (const uint16_t*)q,
               (uint16_t*)C, (uint16_t*)Qp, H, Hp, d, HD, r, row0, T_cap, 4, scale,
               (const uint16_t*)Bm2, (const uint16_t*)x2, (uint16_t*)C2};
  const bool dot = x != nullptr, fold = q != nullptr, pair = Bm2 != nullptr;
  if (pair && !(dot && x2 && C2)) {
    set_error("basis pass: a second append needs a first one and all of Bm2, x2, C2");
    return AP_ERR_INVALID_ARG;
  }
  if (dt == AP_F16) {
    if (pair) return fold ? launch_rows<F16Tag, true, true, true>(p, B, stream) : launch_rows<F16Tag, true, false, true>(p, B, stream);
    if (dot && fold) return launch_rows<F16Tag, true, true, false>(p, B, stream);
    if (dot) return launch_rows<F16Tag, true, false, false>(p, B, stream);
    return launch_rows<F16Tag, false, true, false>(p, B, stream);
  }
  if (pair) return fold ? launch_rows<BF16Tag, true, true, true>(p, B, stream) : launch_rows<BF16Tag, true, false, true>(p, B, stream);
  if (dot && fold) return launch_rows<BF16Tag, true, true, false>(p, B, stream);
  if (dot) return launch_rows<BF16Tag, true, false, false>(p, B, stream);
  return launch_rows<BF16Tag, false, true, false>(p, B, stream);
}

ap_status launch_fold_heads(ap_dtype dt, const void* Bk, int64_t bstride, const void* q, void* Qp, int B,
                            int H, int H_kv, int Hp, int d, int r, float scale, hipStream_t stream) {
  const int G = H / H_kv;
  const dim3 grid(H_kv * ((G + 7) / 8), (r + 63) / 64, B);
#define AP_FH(TAG, L)                                                                                   \
  hipLaunchKernelGGL((fold_heads<TAG, L>), grid, dim3(256), 0, stream, (const uint16_t*)Bk, bstride,    \
                     (const uint16_t*)q, (uint16_t*)Qp, H, G, Hp, r, scale)
  if (dt == AP_F16) {
    switch (d) { case 32: AP_FH(F16Tag, 4); break; case 64: AP_FH(F16Tag, 8); break;
                 case 128: AP_FH(F16Tag, 16); break; default: AP_FH(F16Tag, 32); break; }
  } else {
    switch (d) { case 32: AP_FH(BF16Tag, 4); break; case 64: AP_FH(BF16Tag, 8); break;
                 case 128: AP_FH(BF16Tag, 16); break; default: AP_FH(BF16Tag, 32); break; }
  }
#undef AP_FH
  return AP_OK;
}

int basis_rows_per_wave(int B, int r) {
  // about five workgroups per CU, two of them resident at a time: the start and the end of a
  // workgroup (vector slices in, folded tile out) then overlap other workgroups' streaming
  int rpw = (int)(((int64_t)B * r + 5119) / 5120);
  return rpw < 4 ? 4 : (rpw > 32 ? 32 : rpw);
}
// expand_append: about four two-wave workgroups per CU in one round, but never more than 16 row
// blocks per sequence at large batches (each block writes an HD-wide partial output that
// reduce_out reads back; measured at 64 sequences of rank 640 with the non-temporal row loads:
// 16 blocks 292 us per step, 10 blocks 292, 8 blocks 295, 32 blocks 310, 5 blocks 328); small
// batches, whose partial outputs are small anyway, take up to 64 blocks so that the launch still
// fills the chip.
int expand_rows_per_pair(int B, int r) {
  int rpw = (int)(((int64_t)B * r + 1023) / 1024);
  const int nob_max = B >= 32 ? 16 : B >= 16 ? 32 : 64;
  const int floor_rows = (r + nob_max - 1) / nob_max;
  if (rpw < floor_rows) rpw = floor_rows;
  return rpw < 4 ? 4 : (rpw > 128 ? 128 : rpw);
}

ap_status launch_merge_splits(const float* part_ml, const float* part_U, float* out_ml, float* out_U,
                              float* pnew, const int* pnew_split, int B, int H, int r, int S,
                              hipStream_t stream) {
  const size_t lds = ((size_t)S + 256) * 4;
  hipLaunchKernelGGL(merge_splits, dim3((r + 63) / 64, H, B), dim3(256), lds, stream, part_ml, part_U,
                     out_ml, out_U, pnew, pnew_split, H, r, S);
  return AP_OK;
}
int expand_row_blocks(int B, int r) { return (r + expand_rows_per_pair(B, r) - 1) / expand_rows_per_pair(B, r); }

ap_status launch_expand_append(ap_dtype dt, bool out_f32, const void* Bv, int64_t bstride,
                               const void* v_new, void* Cv, const float* part_ml,
                               const float* part_U, const float* pnew, const int* pnew_split,
                               const int32_t* rank_v, float* pout, void* out,
                               float* lse, int B, int H, int d, int r, int T, int T_cap, int nsplit,
                               hipStream_t stream) {
  ExpandParams p{(const uint16_t*)Bv, bstride, (const uint16_t*)v_new, (uint16_t*)Cv, part_ml, part_U,
                 pnew, pnew_split, rank_v, pout, lse, H, d, H * d, r, T, T_cap, nsplit, expand_rows_per_pair(B, r),
                 expand_row_blocks(B, r)};
  const dim3 grid(p.nob, B);
  const size_t lds = ((size_t)H * (p.rpw + 1) + 3 * (size_t)H + 4 + (nsplit * H <= 4096 ? (size_t)nsplit * H : 0)) * 4;
  const int kpc = (p.HD + 511) / 512;
#define AP_EA(TAG, K, NB)                                                                        \
  if (kpc <= K) {                                                                                \
    hipLaunchKernelGGL((expand_append<TAG, K, NB>), grid, dim3(128), lds, stream, p);            \
    break;                                                                                       \
  }
  do {
    if (dt == AP_F16) { AP_EA(F16Tag, 2, 3) AP_EA(F16Tag, 4, 3) AP_EA(F16Tag, 8, 3) AP_EA(F16Tag, 10, 2) AP_EA(F16Tag, 16, 2) }
    else { AP_EA(BF16Tag, 2, 3) AP_EA(BF16Tag, 4, 3) AP_EA(BF16Tag, 8, 3) AP_EA(BF16Tag, 10, 2) AP_EA(BF16Tag, 16, 2) }
    set_error("expand: H*d=%d exceeds 8192", p.HD);
    return AP_ERR_UNSUPPORTED;
  } while (0);
#undef AP_EA
  const dim3 g2((p.HD + 1023) / 1024, B);
  if (dt == AP_F16) {
    if (out_f32) hipLaunchKernelGGL((reduce_out<F16Tag, true>), g2, dim3(256), 0, stream, pout, out, p.HD, p.nob);
    else hipLaunchKernelGGL((reduce_out<F16Tag, false>), g2, dim3(256), 0, stream, pout, out, p.HD, p.nob);
  } else {
    if (out_f32) hipLaunchKernelGGL((reduce_out<BF16Tag, true>), g2, dim3(256), 0, stream, pout, out, p.HD, p.nob);
    else hipLaunchKernelGGL((reduce_out<BF16Tag, false>), g2, dim3(256), 0, stream, pout, out, p.HD, p.nob);
  }
  return AP_OK;
}

ap_status launch_merge_expand(ap_dtype dt, bool out_f32, const float* part_ml, const float* part_U,
                              const void* Bv, int64_t bstride, void* out, float* lse, int B, int H,
                              int H_kv, int d, int r, int nsplit, hipStream_t stream) {
  const int G = H / H_kv;
  const int rows = 256 / ((2 * d) >> 3);
  const size_t lds = ((size_t)2 * r + (size_t)rows * 2 * d) * 4;
  const dim3 grid((H + 1) / 2, B);
  const uint16_t* bv = (const uint16_t*)Bv;
  if (nsplit > 16) {
    set_error("merge_expand: %d splits (at most 16 are merged inline)", nsplit);
    return AP_ERR_UNSUPPORTED;
  }
#define AP_ME(TAG, F32, KS) \
  hipLaunchKernelGGL((merge_expand<TAG, F32, KS>), grid, dim3(256), lds, stream, part_ml, part_U, bv, bstride, out, lse, H, G, d, r, nsplit)
#define AP_ME_KS(TAG, F32) do { if (nsplit <= 8) AP_ME(TAG, F32, 8); else AP_ME(TAG, F32, 16); } while (0)
  if (dt == AP_F16) {
    if (out_f32) AP_ME_KS(F16Tag, true);
    else AP_ME_KS(F16Tag, false);
  } else {
    if (out_f32) AP_ME_KS(BF16Tag, true);
    else AP_ME_KS(BF16Tag, false);
  }
#undef AP_ME_KS
#undef AP_ME
  return AP_OK;
}

}  // namespace ap
