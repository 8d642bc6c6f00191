// The uncompressed segment of the cache (paper Alg. 1: C_u = {K, V}, the text tokens and the
// tokens generated since the last compression) and the merge of segments under one softmax.
//
//   raw_attn_partial   flash-decode over raw K, V [B, T_u_cap, HD] in 16-bit storage: a
//                      workgroup owns the query heads that share one key/value head (up to
//                      eight; every head alone without grouped queries) of one sequence and
//                      a range of tokens; groups of d/8 lanes take one token each (one
//                      16-byte chunk of the key and value slice per lane, loaded once for all
//                      the heads), several tokens in flight per group, online softmax per
//                      group and head, groups combined through LDS at the end.
//   keyonly_partial    the same flash-decode for a cache whose KEYS are compressed (coefficients
//                      C_k [B, T_cap, r] and a basis) while its values stay raw (appendix "Analysis of
//                      Textual Token Compression": keys only, R_k = 64): the basis is
//                      folded into the query beforehand, a token's score is the dot product
//                      of its coefficient row with the folded query of the head.
//   merge_parts        attention over disjoint token sets -> attention over their union:
//                      out = sum_i w_i out_i / sum_i w_i,  w_i = exp(lse_i - max lse),
//                      lse = max lse + log sum_i w_i  (the partial decompression of Alg. 1
//                      concatenates the segments; a softmax over a concatenation is this
//                      weighted mean of the per-segment softmaxes).
//   raw_append         copy the new token's key and value rows to the end of the segment.
// Sums are fp32; products of two 16-bit values are exact in fp32.
#include "ap_common.hpp"
#include "lane_ops.hpp"

namespace ap {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kUnroll = 4;       // tokens in flight per lane group

// Heads of one workgroup: NQ query heads that share a key/value head (grouped queries), so a
// key or value chunk is loaded once and used NQ times.  A key/value head with QG query heads
// is covered by ceil(QG / NQ) workgroups; the last may hold fewer than NQ heads (its unused
// slots repeat the first head and write nothing).
constexpr int heads_per_wg(int QG) { return QG >= 5 ? 8 : QG >= 3 ? 4 : QG >= 2 ? 2 : 1; }

struct HeadBlock {
  int h0, nq, kvh;
};
template <int NQ>
__device__ __forceinline__ HeadBlock head_block(int idx, int QG) {
  const int nsub = (QG + NQ - 1) / NQ;
  const int kvh = idx / nsub, sub = idx - kvh * nsub;
  int nq = QG - sub * NQ;
  nq = nq < NQ ? nq : NQ;
  return {kvh * QG + sub * NQ, nq, kvh};
}

// The contribution of N tokens to the online softmax of one head: one maximum over the N
// scores, at most one move of the reference exponent (the accumulators are rescaled under a
// branch that is rarely taken after the first tokens), N independent exponentials.
template <int N, int W = 8>
__device__ __forceinline__ void softmax_steps(const float (&s)[N], const bool (&valid)[N], const float (&vf)[N][W],
                                              float& m, float& l, float (&o)[W]) {
  float mx = -INFINITY;
#pragma unroll
  for (int u = 0; u < N; ++u) mx = fmaxf(mx, valid[u] ? s[u] : -INFINITY);
  if (mx > m) {
    const float alpha = fast_exp2(m - mx);               // 0 on the first tokens (m = -inf)
    l *= alpha;
#pragma unroll
    for (int e = 0; e < W; ++e) o[e] *= alpha;
    m = mx;
  }
#pragma unroll
  for (int u = 0; u < N; ++u) {
    const float pw = valid[u] ? fast_exp2(s[u] - m) : 0.f;   // m is finite wherever a token is valid
    l += pw;
#pragma unroll
    for (int e = 0; e < W; ++e) o[e] = fmaf(pw, vf[u][e], o[e]);
  }
}

// 16 bytes of 16-bit values -> eight floats.
template <class Tag>
__device__ __forceinline__ void widen8(const u32x4_t& v, float (&f)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) { f[2 * e] = lo_to_f32(v[e], Tag{}); f[2 * e + 1] = hi_to_f32(v[e], Tag{}); }
}

// The groups of a workgroup hold partial (m, l, o) of the same heads over different tokens:
// combine them through LDS, one head at a time, and write the normalised partial output
// [su][b][h][d] and its log-sum-exp [su][b][h].
template <int LPH, int NQ>
__device__ __forceinline__ void combine_groups(const float (&m)[NQ], const float (&l)[NQ], const float (&o)[NQ][8],
                                               const HeadBlock& hb, int su, int b, int B, int H,
                                               float* __restrict__ out_part, float* __restrict__ lse_part) {
  constexpr int d = LPH * 8;
  constexpr int G = 256 / LPH;
  __shared__ float red[G][d + 2];
  const int tid = threadIdx.x, g = tid / LPH, li = tid % LPH;
#pragma unroll
  for (int k = 0; k < NQ; ++k) {
    if (k < hb.nq) {                                     // same for the whole workgroup
#pragma unroll
      for (int e = 0; e < 8; ++e) red[g][li * 8 + e] = o[k][e];
      if (li == 0) { red[g][d] = m[k]; red[g][d + 1] = l[k]; }
    }
    __syncthreads();
    if (k < hb.nq) {
      float mstar = -INFINITY;
      for (int i = 0; i < G; ++i) mstar = fmaxf(mstar, red[i][d]);
      const size_t po = ((size_t)su * B + b) * H + hb.h0 + k;
      if (mstar == -INFINITY) {                          // no token in this range
        if (tid < d) out_part[po * d + tid] = 0.f;
        if (tid == 0) lse_part[po] = -INFINITY;
      } else if (tid < d) {
        float acc = 0.f, L = 0.f;
        for (int i = 0; i < G; ++i) {
          const float w = fast_exp2(red[i][d] - mstar);  // 0 for a group without tokens
          acc = fmaf(w, red[i][tid], acc);
          L = fmaf(w, red[i][d + 1], L);
        }
        out_part[po * d + tid] = acc / L;
        if (tid == 0) lse_part[po] = (mstar + log2f(L)) * kLn2;
      }
    }
    __syncthreads();
  }
}

// grid (H_kv * ceil(QG / NQ), S, B), 256 threads.  LPH = d / 8 lanes form a group; G = 256 / LPH
// groups.  QG query heads share one key/value head (1 = every head has its own).
// Split su covers tokens [su * per, min(T, (su + 1) * per)); group g takes every G-th of them.
template <class Tag, int LPH, int NQ>
__global__ void __launch_bounds__(256)
raw_attn_partial(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K,
                 const uint16_t* __restrict__ V, float* __restrict__ out_part,
                 float* __restrict__ lse_part, int B, int H, int QG, int T, int T_cap, int per,
                 float scale_log2) {
  constexpr int d = LPH * 8;
  constexpr int G = 256 / LPH;
  const HeadBlock hb = head_block<NQ>(blockIdx.x, QG);
  const int su = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, g = tid / LPH, li = tid % LPH;
  const size_t HD = (size_t)(H / QG) * d;
  u32x4_t qv[NQ];
#pragma unroll
  for (int k = 0; k < NQ; ++k)
    qv[k] = *(const u32x4_t*)(q + ((size_t)b * H + hb.h0 + (k < hb.nq ? k : 0)) * d + li * 8);
  const uint16_t* Kb = K + (size_t)b * T_cap * HD + (size_t)hb.kvh * d + li * 8;
  const uint16_t* Vb = V + (size_t)b * T_cap * HD + (size_t)hb.kvh * d + li * 8;
  const int t0 = su * per;
  int t1 = t0 + per;
  t1 = t1 < T ? t1 : T;

  float m[NQ], l[NQ], o[NQ][8];
#pragma unroll
  for (int k = 0; k < NQ; ++k) {
    m[k] = -INFINITY; l[k] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[k][e] = 0.f;
  }
  // every group runs the same number of rounds; a round's tokens beyond the range are clamped
  // to the last token of the range (an in-bounds repeat) and masked out of the softmax
  const int ntok = t1 - t0;
  const int rounds = ntok > 0 ? (ntok + G * kUnroll - 1) / (G * kUnroll) : 0;
  for (int rd = 0; rd < rounds; ++rd) {
    u32x4_t kv[kUnroll], vv[kUnroll];
    int tok[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      tok[u] = t0 + (rd * kUnroll + u) * G + g;
      const int tc = tok[u] < t1 ? tok[u] : t1 - 1;
      if constexpr (NQ == 1) {
        // every key and value row is read once per launch: non-temporal (60 -> 54 us for 64 x 256
        // tokens at 40 heads; with several query heads per workgroup the hint cost 3 %)
        kv[u] = __builtin_nontemporal_load((const u32x4_t*)(Kb + (size_t)tc * HD));
        vv[u] = __builtin_nontemporal_load((const u32x4_t*)(Vb + (size_t)tc * HD));
      } else {
        kv[u] = *(const u32x4_t*)(Kb + (size_t)tc * HD);
        vv[u] = *(const u32x4_t*)(Vb + (size_t)tc * HD);
      }
    }
    float vf[kUnroll][8];
    bool valid[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      widen8<Tag>(vv[u], vf[u]);
      valid[u] = tok[u] < t1;                            // same decision in all lanes of the group
    }
#pragma unroll
    for (int k = 0; k < NQ; ++k) {
      float sc[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) sc[u] = group_sum<LPH>(dot8<Tag>(kv[u], qv[k], 0.f)) * scale_log2;
      softmax_steps<kUnroll>(sc, valid, vf, m[k], l[k], o[k]);
    }
  }
  combine_groups<LPH, NQ>(m, l, o, hb, su, b, B, H, out_part, lse_part);
}

// Key-only compression.  grid (S, H_kv * ceil(QG / NQ), B), 256 threads; the split index varies
// fastest, and S is a multiple of 8 whenever there is more than one split, so the workgroups
// of all heads that walk one token range sit on the same XCD and find its coefficient rows
// (shared by every head) in that XCD's L2.
// Qp [B][2][H][r]: the folded queries as hi + lo 16-bit pairs, softmax scale and log2(e)
// included.  A group of LPH lanes takes a token: lane li holds the value chunk li and the
// coefficient chunks li, li + LPH, ... (16 bytes each; NCH of them, those at or beyond r / 8
// re-read chunk 0 against a zero query).  KU tokens are in flight per group.
// PAIR (a coefficient row fills at most half a group: r / 8 <= LPH / 2, NCH = 1): the two halves
// of a group score two different tokens at once, each half summing its own row, and swap the
// results; half the score arithmetic and half the coefficient loads per token.
template <class Tag, int LPH, int NCH, int KU, int NQ, bool PAIR>
__global__ void __launch_bounds__(256)
keyonly_partial(const uint16_t* __restrict__ Qp, const uint16_t* __restrict__ Ck,
                const uint16_t* __restrict__ V, float* __restrict__ out_part,
                float* __restrict__ lse_part, int B, int H, int QG, int T, int T_cap, int r, int per) {
  constexpr int d = LPH * 8;
  constexpr int G = 256 / LPH;
  const HeadBlock hb = head_block<NQ>(blockIdx.y, QG);
  const int su = blockIdx.x, b = blockIdx.z;
  const int tid = threadIdx.x, g = tid / LPH, li = tid % LPH;
  const size_t HD = (size_t)(H / QG) * d;
  const int nchunk = r >> 3;
  static_assert(!PAIR || (NCH == 1 && KU % 2 == 0), "pairing needs one chunk per lane and whole pairs");
  constexpr int LS = PAIR ? LPH / 2 : LPH;          // lanes that share a coefficient row
  const int half = PAIR ? li / LS : 0;
  u32x4_t qh[NQ][NCH], ql[NQ][NCH];
  uint32_t coff[NCH];                               // element offset of the lane's chunks in a row
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int kc = (PAIR ? li % LS : li) + LPH * c;
    coff[c] = kc < nchunk ? (uint32_t)kc * 8u : 0u;
#pragma unroll
    for (int k = 0; k < NQ; ++k) {
      const u32x4_t z = {0, 0, 0, 0};
      qh[k][c] = z; ql[k][c] = z;
      if (kc < nchunk) {
        const uint16_t* qp = Qp + (((size_t)b * 2) * H + hb.h0 + (k < hb.nq ? k : 0)) * r + kc * 8;
        qh[k][c] = *(const u32x4_t*)qp;
        ql[k][c] = *(const u32x4_t*)(qp + (size_t)H * r);
      }
    }
  }
  const uint16_t* Cb = Ck + (size_t)b * T_cap * r;
  const uint16_t* Vb = V + (size_t)b * T_cap * HD + (size_t)hb.kvh * d + li * 8;
  const int t0 = su * per;
  int t1 = t0 + per;
  t1 = t1 < T ? t1 : T;

  float m[NQ], l[NQ], o[NQ][8];
#pragma unroll
  for (int k = 0; k < NQ; ++k) {
    m[k] = -INFINITY; l[k] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[k][e] = 0.f;
  }
  const int ntok = t1 - t0;
  const int rounds = ntok > 0 ? (ntok + G * KU - 1) / (G * KU) : 0;
  for (int rd = 0; rd < rounds; ++rd) {
    constexpr int NR = PAIR ? KU / 2 : KU;             // coefficient rows a lane loads per round
    u32x4_t cv[NR][NCH], vv[KU];
    int tok[KU];
    // slot u of a lane holds token (rd KU + u') G + g of the split; u' = u, except that with PAIR
    // the second half of a group swaps the two slots of every pair, so that slot 2p is the
    // token whose coefficient row this lane's half scores
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      tok[u] = t0 + (rd * KU + (PAIR ? u ^ half : u)) * G + g;
      const int tc = tok[u] < t1 ? tok[u] : t1 - 1;      // in-bounds repeat, masked below
      vv[u] = *(const u32x4_t*)(Vb + (size_t)tc * HD);
    }
#pragma unroll
    for (int p = 0; p < NR; ++p) {
      const int tk = tok[PAIR ? 2 * p : p];
      const int tc = tk < t1 ? tk : t1 - 1;
      const uint16_t* crow = Cb + (size_t)tc * r;
#pragma unroll
      for (int c = 0; c < NCH; ++c) cv[p][c] = *(const u32x4_t*)(crow + coff[c]);
    }
    float vf[KU][8];
    bool valid[KU];
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      widen8<Tag>(vv[u], vf[u]);
      valid[u] = tok[u] < t1;                            // same decision in all lanes of the group
    }
#pragma unroll
    for (int k = 0; k < NQ; ++k) {
      float sc[KU];
#pragma unroll
      for (int p = 0; p < NR; ++p) {
        float part = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
          part = dot8<Tag>(cv[p][c], ql[k][c], dot8<Tag>(cv[p][c], qh[k][c], part));
        if constexpr (PAIR) {
          sc[2 * p] = group_sum<LS>(part);               // this half's token: slot 2p
          sc[2 * p + 1] = other_half<LPH>(sc[2 * p]);    // the other half's token: slot 2p + 1
        } else {
          sc[p] = group_sum<LPH>(part);
        }
      }
      softmax_steps<KU>(sc, valid, vf, m[k], l[k], o[k]);
    }
  }
  combine_groups<LPH, NQ>(m, l, o, hb, su, b, B, H, out_part, lse_part);
}

// Value-only compression (raw keys, compressed values): scores as in raw_attn_partial, the
// weighted sum runs over the value COEFFICIENT rows, U[h, j] = sum_t p[h, t] C_v[t, j], and the
// expansion through B_v is left to merge_expand.  grid (S, H_kv * ceil(QG / NQ), B) as for
// key-only compression (the coefficient rows are shared by every head).  Lane li of a group
// holds the key chunk li of a token and the coefficient chunks li, li + LPH, ... (NCH of them),
// i.e. columns [c d + 8 li, c d + 8 li + 8) for c < NCH.  Writes what merge_expand reads: per
// split and head the reference exponent (log2 units) and the sum, part_ml [B][S][H][2], and the
// unnormalised coefficient sums part_U [B][S][H][r].
template <class Tag, int LPH, int NCH, int KU, int NQ>
__global__ void __launch_bounds__(256)
valueonly_partial(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K,
                  const uint16_t* __restrict__ Cv, float* __restrict__ part_ml,
                  float* __restrict__ part_U, int H, int QG, int T, int T_cap, int r, int per,
                  float scale_log2) {
  constexpr int d = LPH * 8;
  constexpr int G = 256 / LPH;
  constexpr int W = NCH * 8;
  __shared__ float red[G][d + 2];
  const HeadBlock hb = head_block<NQ>(blockIdx.y, QG);
  const int su = blockIdx.x, S = gridDim.x, b = blockIdx.z;
  const int tid = threadIdx.x, g = tid / LPH, li = tid % LPH;
  const size_t HD = (size_t)(H / QG) * d;
  const int nchunk = r >> 3;
  u32x4_t qv[NQ];
#pragma unroll
  for (int k = 0; k < NQ; ++k)
    qv[k] = *(const u32x4_t*)(q + ((size_t)b * H + hb.h0 + (k < hb.nq ? k : 0)) * d + li * 8);
  uint32_t coff[NCH];                               // chunks beyond the row re-read chunk 0; never stored
#pragma unroll
  for (int c = 0; c < NCH; ++c) coff[c] = li + LPH * c < nchunk ? (uint32_t)(li + LPH * c) * 8u : 0u;
  const uint16_t* Kb = K + (size_t)b * T_cap * HD + (size_t)hb.kvh * d + li * 8;
  const uint16_t* Cb = Cv + (size_t)b * T_cap * r;
  const int t0 = su * per;
  int t1 = t0 + per;
  t1 = t1 < T ? t1 : T;

  float m[NQ], l[NQ], u[NQ][W];
#pragma unroll
  for (int k = 0; k < NQ; ++k) {
    m[k] = -INFINITY; l[k] = 0.f;
#pragma unroll
    for (int e = 0; e < W; ++e) u[k][e] = 0.f;
  }
  const int ntok = t1 - t0;
  const int rounds = ntok > 0 ? (ntok + G * KU - 1) / (G * KU) : 0;
  for (int rd = 0; rd < rounds; ++rd) {
    u32x4_t kv[KU], cv[KU][NCH];
    bool valid[KU];
#pragma unroll
    for (int t = 0; t < KU; ++t) {
      const int tok = t0 + (rd * KU + t) * G + g;
      valid[t] = tok < t1;                               // same decision in all lanes of the group
      const int tc = valid[t] ? tok : t1 - 1;            // in-bounds repeat, masked in the softmax
      kv[t] = *(const u32x4_t*)(Kb + (size_t)tc * HD);
      const uint16_t* crow = Cb + (size_t)tc * r;
#pragma unroll
      for (int c = 0; c < NCH; ++c) cv[t][c] = *(const u32x4_t*)(crow + coff[c]);
    }
    float cf[KU][W];
#pragma unroll
    for (int t = 0; t < KU; ++t)
#pragma unroll
      for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          cf[t][c * 8 + 2 * e] = lo_to_f32(cv[t][c][e], Tag{});
          cf[t][c * 8 + 2 * e + 1] = hi_to_f32(cv[t][c][e], Tag{});
        }
#pragma unroll
    for (int k = 0; k < NQ; ++k) {
      float sc[KU];
#pragma unroll
      for (int t = 0; t < KU; ++t) sc[t] = group_sum<LPH>(dot8<Tag>(kv[t], qv[k], 0.f)) * scale_log2;
      softmax_steps<KU, W>(sc, valid, cf, m[k], l[k], u[k]);
    }
  }
  // ---- combine the groups: one head and one block of d columns at a time
#pragma unroll
  for (int k = 0; k < NQ; ++k) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      if (k < hb.nq) {                                   // same for the whole workgroup
#pragma unroll
        for (int e = 0; e < 8; ++e) red[g][li * 8 + e] = u[k][c * 8 + e];
        if (li == 0) { red[g][d] = m[k]; red[g][d + 1] = l[k]; }
      }
      __syncthreads();
      if (k < hb.nq && tid < d) {
        float mstar = -INFINITY;
        for (int i = 0; i < G; ++i) mstar = fmaxf(mstar, red[i][d]);
        float acc = 0.f, L = 0.f;
        if (mstar > -INFINITY) {
          for (int i = 0; i < G; ++i) {
            const float w = fast_exp2(red[i][d] - mstar);   // 0 for a group without tokens
            acc = fmaf(w, red[i][tid], acc);
            L = fmaf(w, red[i][d + 1], L);
          }
        }
        const size_t ps = ((size_t)b * S + su) * H + hb.h0 + k;
        const int col = c * d + tid;
        if (col < r) part_U[ps * r + col] = acc;
        if (c == 0 && tid == 0) { part_ml[ps * 2] = mstar; part_ml[ps * 2 + 1] = L; }
      }
      __syncthreads();
    }
  }
}

// Up to kMaxLists lists of parts; list i holds cnt[i] parts, `ostride` floats apart in out and
// `lstride` floats apart in lse (a single [B, H, d] segment is a list of one part).
constexpr int kMaxLists = 2;
struct MergeArgs {
  const float* out[kMaxLists];
  const float* lse[kMaxLists];
  int cnt[kMaxLists];
  size_t ostride, lstride;
};

// grid (ceil(H d / 256), B), 256 threads: one output element per thread.  Parts are taken eight
// at a time so that their loads are in flight together (a list can hold 64 splits).
template <class Tag, bool OUT_F32>
__global__ void __launch_bounds__(256)
merge_parts(const MergeArgs a, void* __restrict__ out, float* __restrict__ lse, int H, int d) {
  const int b = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
  if (i >= H * d) return;
  const int h = i / d;
  const size_t lo = (size_t)b * H + h, oo = (size_t)b * H * d + i;
  float m = -INFINITY;
  for (int k = 0; k < kMaxLists; ++k)
    for (int c0 = 0; c0 < a.cnt[k]; c0 += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = c0 + u < a.cnt[k] ? a.lse[k][lo + (c0 + u) * a.lstride] : -INFINITY;
#pragma unroll
      for (int u = 0; u < 8; ++u) m = fmaxf(m, v[u]);
    }
  float acc = 0.f, z = 0.f;
  if (m > -INFINITY) {
    for (int k = 0; k < kMaxLists; ++k)
      for (int c0 = 0; c0 < a.cnt[k]; c0 += 8) {
        float v[8], x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const bool on = c0 + u < a.cnt[k];
          v[u] = on ? a.lse[k][lo + (c0 + u) * a.lstride] : -INFINITY;
          x[u] = on ? a.out[k][oo + (c0 + u) * a.ostride] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float w = __expf(v[u] - m);               // 0 for an empty part and beyond the list
          acc = fmaf(w, x[u], acc);
          z += w;
        }
      }
    acc /= z;
  }
  if (OUT_F32) ((float*)out)[oo] = acc;
  else ((uint16_t*)out)[oo] = f32_to_bits(acc, Tag{});
  if (lse && i == h * d) lse[lo] = m > -INFINITY ? m + __logf(z) : -INFINITY;
}

// grid (ceil(HD / 2048), B), 256 threads: rows of HD 16-bit elements, 16 bytes per thread.
__global__ void __launch_bounds__(256)
raw_append(const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
           uint16_t* __restrict__ K, uint16_t* __restrict__ V, int HD, int row, int T_cap) {
  const int b = blockIdx.y, e = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (e >= HD) return;
  const size_t src = (size_t)b * HD + e, dst = ((size_t)b * T_cap + row) * HD + e;
  if (k_new) *(u32x4_t*)(K + dst) = *(const u32x4_t*)(k_new + src);
  if (v_new) *(u32x4_t*)(V + dst) = *(const u32x4_t*)(v_new + src);
}

// Splits of the token axis for `wgs` workgroups per split: about two workgroups per CU
// (measured: four per CU are 10 % slower at batch 64, one per CU 25 % slower at batch 8); a
// split holds at least one round of every group.
int raw_splits(int wgs, int d, int T) {
  const int G = 256 / (d / 8);
  int s = (512 + wgs - 1) / wgs;
  const int by_len = (T + G * kUnroll - 1) / (G * kUnroll);
  if (s > by_len) s = by_len;
  if (s > 64) s = 64;
  return s < 1 ? 1 : s;
}
// Workgroups per split: one per block of query heads that share a key/value head.
int raw_wgs(int B, int H, int H_kv) {
  const int QG = H / H_kv, nq = heads_per_wg(QG);
  return B * H_kv * ((QG + nq - 1) / nq);
}
// The workspace query does not know H_kv: it assumes the fewest workgroups per split any H_kv
// can give (eight heads each), hence the most splits.
int raw_splits_most(int B, int H, int d, int T) { return raw_splits(B * ((H + 7) / 8), d, T); }

template <class Tag>
void launch_raw_partial(const void* q, const void* K, const void* V, float* op, float* lp, int B, int H,
                        int QG, int d, int T, int T_cap, int S, float sm_scale, hipStream_t stream) {
  const int per = (T + S - 1) / S;
  const int nq = heads_per_wg(QG);
  const dim3 grid((H / QG) * ((QG + nq - 1) / nq), S, B);
  const float sc = sm_scale * kLog2e;
#define AP_RAW2(L, N)                                                                              \
  hipLaunchKernelGGL((raw_attn_partial<Tag, L, N>), grid, dim3(256), 0, stream, (const uint16_t*)q, \
                     (const uint16_t*)K, (const uint16_t*)V, op, lp, B, H, QG, T, T_cap, per, sc)
#define AP_RAW(L)                                                                                  \
  switch (nq) { case 1: AP_RAW2(L, 1); break; case 2: AP_RAW2(L, 2); break; case 4: AP_RAW2(L, 4); break; \
                default: AP_RAW2(L, 8); break; }
  switch (d) {
    case 32: AP_RAW(4) break;
    case 64: AP_RAW(8) break;
    case 128: AP_RAW(16) break;
    default: AP_RAW(32) break;
  }
#undef AP_RAW
#undef AP_RAW2
}

template <class Tag>
void launch_merge(const MergeArgs& a, void* out, bool out_f32, float* lse, int B, int H, int d,
                  hipStream_t stream) {
  const dim3 grid((H * d + 255) / 256, B);
  if (out_f32) hipLaunchKernelGGL((merge_parts<Tag, true>), grid, dim3(256), 0, stream, a, out, lse, H, d);
  else hipLaunchKernelGGL((merge_parts<Tag, false>), grid, dim3(256), 0, stream, a, out, lse, H, d);
}

// Key-only compression: about four workgroups per CU, a multiple of 8 splits (see the kernel),
// every split at least one round of the widest variant's groups.
int keyonly_heads_per_wg(int QG, int nch) {
  int nq = heads_per_wg(QG);
  const int cap = nch <= 1 ? 8 : nch <= 2 ? 4 : nch <= 3 ? 2 : 1;   // folded queries held in registers
  return nq < cap ? nq : cap;
}
int keyonly_splits(int B, int H, int H_kv, int d, int T, int r) {
  const int LPH = d / 8, G = 256 / LPH, QG = H / H_kv;
  const int nq = keyonly_heads_per_wg(QG, ((r >> 3) + LPH - 1) / LPH);
  const int wgs = B * H_kv * ((QG + nq - 1) / nq);
  int s = (1024 + wgs - 1) / wgs;
  const int by_len = (T + G * 4 - 1) / (G * 4);
  if (s > by_len) s = by_len;
  if (s > 64) s = 64;
  if (s > 1) s = (s + 7) & ~7;
  return s < 1 ? 1 : s;
}

template <class Tag, int LPH>
ap_status launch_keyonly_partial(const uint16_t* Qp, const void* Ck, const void* V, float* op, float* lp,
                                 int B, int H, int QG, int T, int T_cap, int r, int S, hipStream_t stream) {
  const int per = (T + S - 1) / S;
  const int nch = ((r >> 3) + LPH - 1) / LPH;          // 16-byte coefficient chunks per lane
  const int nq = keyonly_heads_per_wg(QG, nch);
  const dim3 grid(S, (H / QG) * ((QG + nq - 1) / nq), B);
#define AP_KO3(N, U, Q, P)                                                                           \
  hipLaunchKernelGGL((keyonly_partial<Tag, LPH, N, U, Q, P>), grid, dim3(256), 0, stream, Qp,        \
                     (const uint16_t*)Ck, (const uint16_t*)V, op, lp, B, H, QG, T, T_cap, r, per)
#define AP_KO2(N, U, Q) AP_KO3(N, U, Q, false)
  if (nch <= 1 && 2 * (r >> 3) <= LPH) {               // a row fills half a group: score tokens in pairs
    switch (nq) { case 1: AP_KO3(1, 4, 1, true); break; case 2: AP_KO3(1, 4, 2, true); break;
                  case 4: AP_KO3(1, 4, 4, true); break; default: AP_KO3(1, 2, 8, true); break; }
    return AP_OK;
  }
  if (nch <= 1) {
    switch (nq) { case 1: AP_KO2(1, 4, 1); break; case 2: AP_KO2(1, 4, 2); break; case 4: AP_KO2(1, 4, 4); break;
                  default: AP_KO2(1, 2, 8); break; }
    return AP_OK;
  }
  if (nch <= 2) {
    switch (nq) { case 1: AP_KO2(2, 4, 1); break; case 2: AP_KO2(2, 4, 2); break; default: AP_KO2(2, 2, 4); break; }
    return AP_OK;
  }
  if (nch <= 3) {
    if (nq == 1) AP_KO2(3, 2, 1); else AP_KO2(3, 2, 2);
    return AP_OK;
  }
  if constexpr (LPH <= 16) { if (nch <= 5) { AP_KO2(5, 2, 1); return AP_OK; } }
  if constexpr (LPH <= 8) { if (nch <= 10) { AP_KO2(10, 1, 1); return AP_OK; } }
  if constexpr (LPH <= 4) { if (nch <= 20) { AP_KO2(20, 1, 1); return AP_OK; } }
#undef AP_KO2
#undef AP_KO3
  set_error("ap_keyonly_attn: r=%d too large for d=%d", r, LPH * 8);
  return AP_ERR_UNSUPPORTED;
}

// Value-only compression: heads per workgroup (their coefficient sums live in registers),
// splits as for key-only compression.
int valueonly_heads_per_wg(int QG, int nch) {
  int nq = heads_per_wg(QG);
  const int cap = nch <= 1 ? 8 : nch <= 2 ? 4 : nch <= 3 ? 2 : 1;
  return nq < cap ? nq : cap;
}
int valueonly_splits(int B, int H, int H_kv, int d, int T, int r) {
  const int LPH = d / 8, G = 256 / LPH, QG = H / H_kv;
  const int nq = valueonly_heads_per_wg(QG, ((r >> 3) + LPH - 1) / LPH);
  const int wgs = B * H_kv * ((QG + nq - 1) / nq);
  int s = (1024 + wgs - 1) / wgs;
  const int by_len = (T + G * 4 - 1) / (G * 4);
  if (s > by_len) s = by_len;
  if (s > 64) s = 64;
  if (s > 1) s = (s + 7) & ~7;
  return s < 1 ? 1 : s;
}

template <class Tag, int LPH>
ap_status launch_valueonly_partial(const void* q, const void* K, const void* Cv, float* ml, float* U, int B,
                                   int H, int QG, int T, int T_cap, int r, int S, float sm_scale,
                                   hipStream_t stream) {
  const int per = (T + S - 1) / S;
  const int nch = ((r >> 3) + LPH - 1) / LPH;
  const int nq = valueonly_heads_per_wg(QG, nch);
  const dim3 grid(S, (H / QG) * ((QG + nq - 1) / nq), B);
  const float sc = sm_scale * kLog2e;
#define AP_VO(N, U_, Q)                                                                             \
  hipLaunchKernelGGL((valueonly_partial<Tag, LPH, N, U_, Q>), grid, dim3(256), 0, stream,           \
                     (const uint16_t*)q, (const uint16_t*)K, (const uint16_t*)Cv, ml, U, H, QG, T,  \
                     T_cap, r, per, sc)
  if (nch <= 1) {
    switch (nq) { case 1: AP_VO(1, 4, 1); break; case 2: AP_VO(1, 4, 2); break; case 4: AP_VO(1, 4, 4); break;
                  default: AP_VO(1, 2, 8); break; }
    return AP_OK;
  }
  if (nch <= 2) {
    switch (nq) { case 1: AP_VO(2, 2, 1); break; case 2: AP_VO(2, 2, 2); break; default: AP_VO(2, 2, 4); break; }
    return AP_OK;
  }
  if (nch <= 3) {
    if (nq == 1) AP_VO(3, 1, 1); else AP_VO(3, 1, 2);
    return AP_OK;
  }
  if constexpr (LPH <= 16) { if (nch <= 5) { AP_VO(5, 1, 1); return AP_OK; } }
  if constexpr (LPH <= 8) { if (nch <= 10) { AP_VO(10, 1, 1); return AP_OK; } }
#undef AP_VO
  set_error("ap_valueonly_attn: r=%d too large for d=%d", r, LPH * 8);
  return AP_ERR_UNSUPPORTED;
}

}  // namespace

size_t raw_attn_workspace(int B, int H, int d, int T) {
  const int S = raw_splits_most(B, H, d, T);
  return round_up((size_t)S * B * H * d * 4, 256) + round_up((size_t)S * B * H * 4, 256);
}

ap_status launch_raw_attn(const void* q, const void* K, const void* V, float* out, float* lse, int B,
                          int H, int H_kv, int d, int T, int T_cap, float sm_scale, ap_dtype dt,
                          void* workspace, hipStream_t stream) {
  const int G = H / H_kv;
  const int S = raw_splits(raw_wgs(B, H, H_kv), d, T);        // never more than the workspace query assumes
  float* op = out;
  float* lp = lse;
  if (S > 1 || !lse) {                     // partial results (or an unwanted lse) go to the workspace
    op = S > 1 ? (float*)workspace : out;
    lp = (float*)((char*)workspace + round_up((size_t)S * B * H * d * 4, 256));
  }
  if (dt == AP_F16) launch_raw_partial<F16Tag>(q, K, V, op, lp, B, H, G, d, T, T_cap, S, sm_scale, stream);
  else launch_raw_partial<BF16Tag>(q, K, V, op, lp, B, H, G, d, T, T_cap, S, sm_scale, stream);
  if (S > 1) {
    MergeArgs a{{op, nullptr}, {lp, nullptr}, {S, 0}, (size_t)B * H * d, (size_t)B * H};
    launch_merge<F16Tag>(a, out, true, lse, B, H, d, stream);
  }
  return check_launch("ap_raw_attn");
}

static size_t keyonly_qp_bytes(int B, int H, int r) { return round_up((size_t)B * 2 * H * r * 2, 256); }

// parts of a key-only call: the matrix-core kernel writes four per split (one per wave)
static int keyonly_parts(int B, int H, int H_kv, int d, int T, int r) {
  return keyonly_mfma_applies(H, H_kv, d, r) ? 4 * keyonly_mfma_splits(B, H_kv, T)
                                             : keyonly_splits(B, H, H_kv, d, T, r);
}

size_t keyonly_attn_workspace(int B, int H, int H_kv, int d, int T, int r) {
  const int P = keyonly_parts(B, H, H_kv, d, T, r);
  return keyonly_qp_bytes(B, H, r) + round_up((size_t)P * B * H * d * 4, 256) +
         round_up((size_t)P * B * H * 4, 256);
}

ap_status launch_keyonly_attn(const void* q, const void* Ck, const void* Bk, int64_t bstride, const void* V,
                              float* out, float* lse, int B, int H, int H_kv, int d, int T, int T_cap, int r,
                              float sm_scale, ap_dtype dt, void* workspace, hipStream_t stream) {
  const int QG = H / H_kv;
  const bool mfma = keyonly_mfma_applies(H, H_kv, d, r);
  const int P = keyonly_parts(B, H, H_kv, d, T, r);
  char* ws = (char*)workspace;
  uint16_t* Qp = (uint16_t*)ws;
  float* parts = (float*)(ws + keyonly_qp_bytes(B, H, r));
  float* lparts = (float*)(ws + keyonly_qp_bytes(B, H, r) + round_up((size_t)P * B * H * d * 4, 256));
  // q' = scale * log2(e) * B_k[:, slice] q_h for every head, written as hi + lo pairs
  ap_status st = launch_fold_heads(dt, Bk, bstride, q, Qp, B, H, H_kv, H, d, r, sm_scale * kLog2e, stream);
  if (st != AP_OK) return st;
  float* op = P > 1 ? parts : out;
  float* lp = (P > 1 || !lse) ? lparts : lse;
  if (mfma) {
    st = launch_keyonly_mfma(dt, Qp, Ck, V, op, lp, B, H, H_kv, T, T_cap, r, P / 4, stream);
  } else {
#define AP_KL(TAG)                                                                                          \
  switch (d) {                                                                                              \
    case 32: st = launch_keyonly_partial<TAG, 4>(Qp, Ck, V, op, lp, B, H, QG, T, T_cap, r, P, stream); break;  \
    case 64: st = launch_keyonly_partial<TAG, 8>(Qp, Ck, V, op, lp, B, H, QG, T, T_cap, r, P, stream); break;  \
    case 128: st = launch_keyonly_partial<TAG, 16>(Qp, Ck, V, op, lp, B, H, QG, T, T_cap, r, P, stream); break; \
    default: st = launch_keyonly_partial<TAG, 32>(Qp, Ck, V, op, lp, B, H, QG, T, T_cap, r, P, stream); break; \
  }
    if (dt == AP_F16) { AP_KL(F16Tag) } else { AP_KL(BF16Tag) }
#undef AP_KL
  }
  if (st != AP_OK) return st;
  if (P > 1) {
    MergeArgs a{{op, nullptr}, {lp, nullptr}, {P, 0}, (size_t)B * H * d, (size_t)B * H};
    launch_merge<F16Tag>(a, out, true, lse, B, H, d, stream);
  }
  return check_launch("ap_keyonly_attn");
}

// value-only compression: [part_ml | part_U | merged ml | merged U (only with more than 8 splits)]
constexpr int kValueOnlyInlineSplits = 8;               // what merge_expand merges by itself
struct ValueOnlyWs { size_t ml, u, mml, mu, total; };
static ValueOnlyWs valueonly_layout(int B, int H, int H_kv, int d, int T, int r) {
  const int S = valueonly_splits(B, H, H_kv, d, T, r);
  ValueOnlyWs w;
  size_t off = 0;
  w.ml = off; off += round_up((size_t)B * S * H * 2 * 4, 256);
  w.u = off; off += round_up((size_t)B * S * H * r * 4, 256);
  w.mml = off; off += round_up((size_t)B * H * 2 * 4, 256);
  w.mu = off; off += S > kValueOnlyInlineSplits ? round_up((size_t)B * H * r * 4, 256) : 0;
  w.total = off;
  return w;
}
size_t valueonly_attn_workspace(int B, int H, int H_kv, int d, int T, int r) {
  return valueonly_layout(B, H, H_kv, d, T, r).total;
}
bool valueonly_rank_ok(int d, int r) { return r <= (d >= 128 ? 640 : d == 64 ? 640 : 320); }

ap_status launch_valueonly_attn(const void* q, const void* K, const void* Cv, const void* Bv, int64_t bstride,
                                float* out, float* lse, int B, int H, int H_kv, int d, int T, int T_cap, int r,
                                float sm_scale, ap_dtype dt, void* workspace, hipStream_t stream) {
  const int QG = H / H_kv;
  const int S = valueonly_splits(B, H, H_kv, d, T, r);
  const ValueOnlyWs w = valueonly_layout(B, H, H_kv, d, T, r);
  char* ws = (char*)workspace;
  float* ml = (float*)(ws + w.ml);
  float* U = (float*)(ws + w.u);
  ap_status st = AP_OK;
#define AP_VL(TAG)                                                                                            \
  switch (d) {                                                                                                \
    case 32: st = launch_valueonly_partial<TAG, 4>(q, K, Cv, ml, U, B, H, QG, T, T_cap, r, S, sm_scale, stream); break;   \
    case 64: st = launch_valueonly_partial<TAG, 8>(q, K, Cv, ml, U, B, H, QG, T, T_cap, r, S, sm_scale, stream); break;   \
    case 128: st = launch_valueonly_partial<TAG, 16>(q, K, Cv, ml, U, B, H, QG, T, T_cap, r, S, sm_scale, stream); break; \
    default: st = launch_valueonly_partial<TAG, 32>(q, K, Cv, ml, U, B, H, QG, T, T_cap, r, S, sm_scale, stream); break;  \
  }
  if (dt == AP_F16) { AP_VL(F16Tag) } else { AP_VL(BF16Tag) }
#undef AP_VL
  if (st != AP_OK) return st;
  int S_exp = S;
  if (S > kValueOnlyInlineSplits) {
    float* ml1 = (float*)(ws + w.mml);
    float* U1 = (float*)(ws + w.mu);
    st = launch_merge_splits(ml, U, ml1, U1, nullptr, nullptr, B, H, r, S, stream);
    if (st != AP_OK) return st;
    ml = ml1; U = U1; S_exp = 1;
  }
  st = launch_merge_expand(dt, true, ml, U, Bv, bstride, out, lse, B, H, H_kv, d, r, S_exp, stream);
  if (st != AP_OK) return st;
  return check_launch("ap_valueonly_attn");
}

ap_status launch_merge_segments(const float* out_a, const float* lse_a, const float* out_b,
                                const float* lse_b, void* out, float* lse, int B, int H, int d,
                                ap_dtype dt_out, hipStream_t stream) {
  MergeArgs a{{out_a, out_b}, {lse_a, lse_b}, {1, 1}, 0, 0};
  if (dt_out == AP_BF16) launch_merge<BF16Tag>(a, out, false, lse, B, H, d, stream);
  else launch_merge<F16Tag>(a, out, dt_out == AP_F32, lse, B, H, d, stream);
  return check_launch("ap_merge_segments");
}

ap_status launch_raw_append(const void* k_new, const void* v_new, void* K, void* V, int B, int HD, int row,
                            int T_cap, hipStream_t stream) {
  hipLaunchKernelGGL(raw_append, dim3((HD + 2047) / 2048, B), dim3(256), 0, stream, (const uint16_t*)k_new,
                     (const uint16_t*)v_new, (uint16_t*)K, (uint16_t*)V, HD, row, T_cap);
  return check_launch("ap_raw_append");
}

}  // namespace ap
