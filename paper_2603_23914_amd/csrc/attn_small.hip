// attn_small: the coefficient-streaming kernel for small ranks (r = 64 or 128, 16-bit storage,
// uniform or per-token ranks), the paper's own operating point (R = 64 ... 128, low group 16).
//
// attn_partial splits a tile of 32 tokens over eight waves in two roles, which costs two
// workgroup barriers and an LDS round trip of the scores per tile: at small ranks its tile loop
// is bound by that dependency chain, not by memory.  Here every wave works alone on whole tiles:
//   scores   S[token, head] = C_k[token, :r] . q'[head, :r]   MFMA 16x16x32, coefficient rows
//            straight from global memory into the A operand, q' (hi + lo) resident as B
//            operands for all MT head tiles;
//   softmax  the MFMA result has the layout of the next product's B operand (lane (head, g)
//            holds tokens 4g..4g+3 and 16+4g..16+4g+3): the weights stay in registers;
//   sums     U^T[column, head] += C_v^T[column, token] . P^T[token, head]: the wave's C_v tile
//            (32 rows of 2r bytes) goes through a private, padded LDS region and is read back
//            as dwords of eight token rows, transposed with byte permutes.
// The four waves of a workgroup take every fourth tile of the split and keep their own
// (reference exponent, sum, U); at the end they are combined through LDS, one wave after the
// other (a fixed order: the result is deterministic), and written in the partial-result layout
// of attn_partial, so the merge and expansion kernels behind it are the same.
#include "ap_common.hpp"
#include "lane_ops.hpp"
#include "mfma_ops.hpp"
#include <hip/hip_ext.h>
#include <type_traits>

namespace ap {
namespace {

constexpr int kTok = 32;
constexpr int kWaves = 4;
constexpr int kTileBytesMax = kTok * (2 * 128 + 16);     // a wave's LDS region (r = 128)

// Registers are capped for two waves per SIMD where a wave's q' and U (all heads) leave room
// for it without spilling (rank 64 up to 48 heads, rank 128 up to 16 heads): measured 5-7 %
// faster there, 25 % slower where the cap forces spills.
#define AP_SMALL_WPE (MT * NKS <= 6 ? 2 : 1)

struct SmallParams {
  const uint16_t* Qp;   // [B][2][Hp][r] folded queries, hi + lo
  const uint16_t* Ck;   // [B][T_cap][r]
  const uint16_t* Cv;
  float* part_ml;       // [B][S][H][2]
  float* part_U;        // [B][S][H][r]
  float* pnew;          // [B][H] weight of the deferred newest token (fused step)
  float* scores;        // [B][T_cap][H] scaled logits in natural-log units, or null
  int B, T, T_cap, r, H, nsplit, xcd_aware, defer_v;
  // per-token ranks (RAGGED): the group lists of ap_select_ranks and the rank arrays
  const int32_t* rank_k;      // [B][T] or null (= r)
  const int32_t* rank_v;
  const int32_t* bucket_off;  // [B][F+1]
  const int32_t* bucket_idx;  // [B][T]
  int F;
};
constexpr int kMaxSmallTiles = 136;     // tiles a split can own with per-token ranks (128 + one per group)

// RAGGED (per-token ranks): a tile is 32 tokens of ONE rank group, taken from the group's index
// list, so the rank is uniform inside a tile; tiles are dealt to the splits round-robin (tile su,
// su + S, ...), as in attn_partial.  The workgroup first writes (token count, key rank, value rank,
// list position) of its tiles into LDS; a wave then gathers a tile's rows through the index
// list.  Columns at or beyond a tile's rank are not fetched (their loads are redirected to the
// row's first chunk) and enter the products as zeros.
template <class Tag, int MT, int NKS, bool RAGGED>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(AP_SMALL_WPE)))
attn_small(const SmallParams p) {
  constexpr int Hp = MT * 16;
  // bf16 carries 8 significant bits: folded queries and weights go to the matrix cores as hi + lo
  // pairs; fp16 (11 bits) needs no second half, as in attn_partial
  constexpr bool SPLIT = std::is_same<Tag, BF16Tag>::value;
  constexpr int R = NKS * 32;                        // the rank, a multiple of 32
  constexpr int CPR = R / 8;                         // 16-byte chunks per coefficient row
  constexpr int NV = CPR / 2;                        // value chunks per lane and tile (32 rows / 64 lanes)
  constexpr int kPitch = 2 * R + 16;                 // LDS row pitch: consecutive row quads on different banks
  constexpr int kDepth = 1;                          // tiles in flight per wave (two measured no faster)
  __shared__ __attribute__((aligned(16))) char vt[kWaves][kTileBytesMax];
  __shared__ float st_m[kWaves][Hp], st_l[kWaves][Hp], st_p[kWaves][Hp];
  static_assert(kWaves * kTileBytesMax >= Hp * R * 4, "the combine buffer reuses the tile regions");
  __shared__ int meta[RAGGED ? kMaxSmallTiles : 1][4];

  const int id = __builtin_amdgcn_readfirstlane((int)blockIdx.x);
  int b, su;
  if (p.xcd_aware) {                                 // a sequence's splits are neighbours on one XCD
    const int k = id >> 3;
    b = (k / p.nsplit) * 8 + (id & 7);
    su = k - (k / p.nsplit) * p.nsplit;
  } else {
    b = id / p.nsplit;
    su = id - b * p.nsplit;
  }
  if (b >= p.B) return;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, n = lane & 15, g = lane >> 4;
  const int T = p.T, H = p.H, S = p.nsplit;
  const int Tv = T - p.defer_v;                      // value rows that exist

  // folded queries: B operand of the score product, lane (head n of tile mt, g): columns 32 ks + 8 g ..
  u32x4_t qh[NKS][MT], ql[SPLIT ? NKS : 1][MT];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const uint16_t* qp = p.Qp + (((size_t)b * 2) * Hp + mt * 16 + n) * R + ks * 32 + g * 8;
      qh[ks][mt] = *(const u32x4_t*)qp;
      if (SPLIT) ql[ks][mt] = *(const u32x4_t*)(qp + (size_t)Hp * R);
    }
  float* logits = p.scores ? p.scores + (size_t)b * H * p.T_cap : nullptr;
  const uint16_t* Cb = p.Ck + (size_t)b * p.T_cap * R + g * 8;
  const uint16_t* Vb = p.Cv + (size_t)b * p.T_cap * R;
  // tiles of this split (the same cuts as attn_partial's)
  int t_lo = 0, ntl = 0;
  const int32_t* bidx = nullptr;
  if constexpr (!RAGGED) {
    const int ntiles = (T + kTok - 1) / kTok;
    t_lo = (int)(((int64_t)su * ntiles) / S);
    ntl = (int)(((int64_t)(su + 1) * ntiles) / S) - t_lo;
  } else {
    const int F = p.F;
    const int32_t* boff = p.bucket_off + (size_t)b * (F + 1);
    bidx = p.bucket_idx + (size_t)b * T;
    int off[9], ts[9];                               // group f: list positions off[f]..off[f+1], first tile ts[f]
    off[0] = boff[0];
    ts[0] = 0;
#pragma unroll
    for (int f = 0; f < 8; ++f) {
      off[f + 1] = f < F ? boff[f + 1] : off[f];
      int c = off[f + 1] - off[f];
      c = c < 0 ? 0 : c;
      ts[f + 1] = ts[f] + ((c + kTok - 1) >> 5);
    }
    const int ntot = ts[8];
    ntl = su < ntot ? (ntot - su + S - 1) / S : 0;
    ntl = ntl < kMaxSmallTiles ? ntl : kMaxSmallTiles;   // the host sizes the splits so that this never cuts
    for (int i = threadIdx.x; i < ntl; i += 256) {
      const int j = su + i * S;
      int o0 = off[0], o1 = off[1], tf = 0;
#pragma unroll
      for (int f = 1; f < 8; ++f)
        if (f < F && j >= ts[f]) { o0 = off[f]; o1 = off[f + 1]; tf = ts[f]; }
      int pos0 = o0 + (j - tf) * kTok;
      int cnt = o1 - pos0;
      cnt = cnt > kTok ? kTok : cnt;
      pos0 = pos0 < 0 ? 0 : (pos0 < T ? pos0 : T - 1);
      cnt = cnt < 1 ? 1 : (pos0 + cnt > T ? T - pos0 : cnt);   // inconsistent lists stay inside the buffers
      int tok = bidx[pos0];
      tok = tok < 0 ? 0 : (tok < T ? tok : T - 1);
      int rk = p.rank_k ? p.rank_k[(size_t)b * T + tok] : R;
      int rv = p.rank_v ? p.rank_v[(size_t)b * T + tok] : R;
      meta[i][0] = cnt;
      meta[i][1] = rk < 0 ? 0 : (rk < R ? rk : R);
      meta[i][2] = rv < 0 ? 0 : (rv < R ? rv : R);
      meta[i][3] = pos0;
    }
    __syncthreads();
  }

  // a tile's rows in registers, and (RAGGED) the token indices of the NEXT tile's rows
  struct TileRegs { u32x4_t A[NKS][2]; u32x4_t Vr[NV]; };
  int tokA[2] = {0, 0}, tokV[NV], tokS[8];           // rows of the A operand, of the value chunks, of the score slots
#pragma unroll
  for (int k2 = 0; k2 < NV; ++k2) tokV[k2] = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) tokS[e] = 0;
  auto fetch_idx = [&](int lt) {                     // RAGGED: token indices of local tile lt for this lane
    const int cnt = __builtin_amdgcn_readfirstlane(meta[lt][0]);
    const int32_t* lst = bidx + __builtin_amdgcn_readfirstlane(meta[lt][3]);
    auto at = [&](int slot) {
      int tok = lst[slot < cnt ? slot : cnt - 1];    // slots beyond the tile repeat its last token (masked)
      return tok < 0 ? 0 : (tok < T ? tok : T - 1);
    };
    tokA[0] = at(n);
    tokA[1] = at(16 + n);
#pragma unroll
    for (int k2 = 0; k2 < NV; ++k2) tokV[k2] = at((lane + 64 * k2) / CPR);
    if (logits) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { tokS[e] = at(4 * g + e); tokS[4 + e] = at(16 + 4 * g + e); }
    }
  };
  auto load_tile = [&](TileRegs& tr, int lt) {
    u32x4_t (&A)[NKS][2] = tr.A;
    u32x4_t (&Vr)[NV] = tr.Vr;
    if constexpr (!RAGGED) {
      const int base = (t_lo + lt) * kTok;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        int row = base + 16 * tt + n;
        row = row < T ? row : T - 1;                 // rows beyond T are masked in the softmax
        const uint16_t* crow = Cb + (size_t)row * R;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) A[ks][tt] = *(const u32x4_t*)(crow + ks * 32);
      }
#pragma unroll
      for (int k2 = 0; k2 < NV; ++k2) {
        const int c = lane + 64 * k2;
        int row = base + c / CPR;
        row = row < Tv ? row : Tv - 1;               // rows that do not exist repeat the last that does
        Vr[k2] = *(const u32x4_t*)(Vb + (size_t)row * R + (c % CPR) * 8);
      }
    } else {
      const int rk = __builtin_amdgcn_readfirstlane(meta[lt][1]);
      const int rv = __builtin_amdgcn_readfirstlane(meta[lt][2]);
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const uint16_t* crow = Cb + (size_t)tokA[tt] * R;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
          A[ks][tt] = *(const u32x4_t*)(crow + (ks * 32 + g * 8 < rk ? ks * 32 : -g * 8));
      }
#pragma unroll
      for (int k2 = 0; k2 < NV; ++k2) {
        const int cc = (lane + 64 * k2) % CPR;
        Vr[k2] = *(const u32x4_t*)(Vb + (size_t)tokV[k2] * R + (cc * 8 < rv ? cc * 8 : 0));
      }
    }
  };

  float m[MT], l[MT], pd[MT];
  f32x4_t U[NKS][2][MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    m[mt] = -INFINITY; l[mt] = 0.f; pd[mt] = 0.f;
#pragma unroll
    for (int i = 0; i < NKS; ++i) { const f32x4_t z = {0.f, 0.f, 0.f, 0.f}; U[i][0][mt] = z; U[i][1][mt] = z; }
  }
  char* my = vt[wave];

  auto process = [&](TileRegs& tr, int lt) {
    u32x4_t (&A)[NKS][2] = tr.A;
    u32x4_t (&Vr)[NV] = tr.Vr;
    const int base = (t_lo + lt) * kTok;               // (not RAGGED) first token of the tile
    // tokens of this tile that exist (>= 1; without per-token ranks it may exceed 32)
    const int cnt = RAGGED ? __builtin_amdgcn_readfirstlane(meta[lt][0]) : T - base;
    const int rk = RAGGED ? __builtin_amdgcn_readfirstlane(meta[lt][1]) : R;
    const int rv = RAGGED ? __builtin_amdgcn_readfirstlane(meta[lt][2]) : R;
    const int slot_new = !RAGGED && p.defer_v ? T - 1 - base : -1;  // the deferred token's slot, if in [0, 32)
    int tokC[8];                                       // RAGGED: this tile's tokens of the lane's score slots
    if constexpr (RAGGED) {
#pragma unroll
      for (int e = 0; e < 8; ++e) tokC[e] = tokS[e];
      if (lt + kWaves < ntl) fetch_idx(lt + kWaves);   // indices of the next tile's rows, used below
    }
#pragma unroll
    for (int k2 = 0; k2 < NV; ++k2) {
      const int c = lane + 64 * k2;
      u32x4_t v = Vr[k2];
      if (RAGGED && (c % CPR) * 8 >= rv) { const u32x4_t z = {0, 0, 0, 0}; v = z; }   // beyond the value rank
      *(u32x4_t*)(my + (c / CPR) * kPitch + (c % CPR) * 16) = v;
    }
    if constexpr (RAGGED) {                            // columns beyond the key rank count as zero
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks)
        if (ks * 32 + g * 8 >= rk) { const u32x4_t z = {0, 0, 0, 0}; A[ks][0] = z; A[ks][1] = z; }
    }
    f32x4_t sp[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
        sp[mt][tt] = z;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          sp[mt][tt] = Mfma<Tag>::run(A[ks][tt], qh[ks][mt], sp[mt][tt]);
          if (SPLIT) sp[mt][tt] = Mfma<Tag>::run(A[ks][tt], ql[ks][mt], sp[mt][tt]);
        }
      }
    if (lt + kDepth * kWaves < ntl) load_tile(tr, lt + kDepth * kWaves);   // the registers are free again
    // ---- softmax of head 16 mt + n: this lane holds tokens 4g+e (tt = 0) and 16+4g+e (tt = 1)
    u32x4_t Phi[MT], Plo[SPLIT ? MT : 1];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float s[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s[e] = 4 * g + e < cnt ? sp[mt][0][e] : -INFINITY;
        s[4 + e] = 16 + 4 * g + e < cnt ? sp[mt][1][e] : -INFINITY;
      }
      if (logits && mt * 16 + n < H) {
        // logits out, for importance tracking: [token][head], so the sixteen lanes of a row group
        // write 64 contiguous bytes per token, also when the tile's tokens are gathered
        float* hcol = logits + (mt * 16 + n);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int ta = RAGGED ? tokC[e] : base + 4 * g + e;
          const int tb = RAGGED ? tokC[4 + e] : base + 16 + 4 * g + e;
          if (4 * g + e < cnt) hcol[(size_t)ta * H] = s[e] * kLn2;
          if (16 + 4 * g + e < cnt) hcol[(size_t)tb * H] = s[4 + e] * kLn2;
        }
      }
      float tmax = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));        // finite: the tile's first token exists
      if (tmax > m[mt]) {                              // same decision in the four lanes of a head
        const float alpha = fast_exp2(m[mt] - tmax);   // 0 on the first tile (m = -inf)
        m[mt] = tmax;
        l[mt] *= alpha;
#pragma unroll
        for (int i = 0; i < NKS; ++i) { U[i][0][mt] *= alpha; U[i][1][mt] *= alpha; }
      }
      float pw[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pw[e] = fast_exp2(s[e] - m[mt]);
      if (slot_new >= 0 && slot_new < kTok && g == ((slot_new >> 2) & 3)) {
        // the newest token's value row does not exist yet: its weight counts in the sum, is
        // exported, and stays out of the products (the expansion pass adds its contribution)
        const int e = (slot_new >> 4) * 4 + (slot_new & 3);
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (k == e) { pd[mt] = pw[k]; pw[k] = 0.f; }
        l[mt] += pd[mt];
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        Phi[mt][c] = cvt_pack(pw[2 * c], pw[2 * c + 1], Tag{});
        float k0 = lo_to_f32(Phi[mt][c], Tag{}), k1 = hi_to_f32(Phi[mt][c], Tag{});
        if (SPLIT) {
          Plo[mt][c] = cvt_pack(pw[2 * c] - k0, pw[2 * c + 1] - k1, Tag{});
          k0 += lo_to_f32(Plo[mt][c], Tag{});
          k1 += hi_to_f32(Plo[mt][c], Tag{});
        }
        l[mt] += k0 + k1;                                // the sum uses the values the MFMA will see
      }
    }
    // ---- U^T += C_v^T . P^T, 32 columns (16 dwords) at a time
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the tile is in LDS for every lane of the wave
    const char* vA = my + (4 * g) * kPitch + n * 4;
    const char* vB = vA + 16 * kPitch;
#pragma unroll
    for (int i = 0; i < NKS; ++i) {
      if (RAGGED && i * 32 >= rv) continue;              // columns beyond the value rank: nothing to add
      uint32_t v[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] = *(const uint32_t*)(vA + e * kPitch + i * 64);
        v[4 + e] = *(const uint32_t*)(vB + e * kPitch + i * 64);
      }
      u32x4_t te, to;                                    // even / odd column of the eight tokens
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        te[c] = __builtin_amdgcn_perm(v[2 * c + 1], v[2 * c], 0x05040100u);
        to[c] = __builtin_amdgcn_perm(v[2 * c + 1], v[2 * c], 0x07060302u);
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        U[i][0][mt] = Mfma<Tag>::run(te, Phi[mt], U[i][0][mt]);
        U[i][1][mt] = Mfma<Tag>::run(to, Phi[mt], U[i][1][mt]);
        if (SPLIT) {
          U[i][0][mt] = Mfma<Tag>::run(te, Plo[mt], U[i][0][mt]);
          U[i][1][mt] = Mfma<Tag>::run(to, Plo[mt], U[i][1][mt]);
        }
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next tile is written
  };
  TileRegs tr0, tr1;
  if (RAGGED && wave < ntl) fetch_idx(wave);
  if (wave < ntl) load_tile(tr0, wave);
  if (kDepth > 1 && wave + kWaves < ntl) load_tile(tr1, wave + kWaves);
  for (int lt = wave; lt < ntl; lt += kDepth * kWaves) {
    process(tr0, lt);
    if (kDepth > 1 && lt + kWaves < ntl) process(tr1, lt + kWaves);
  }

  // ---- combine the four waves: statistics first, then the sums, one wave after the other
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float lt2 = l[mt] + __shfl_xor(l[mt], 16);
    lt2 += __shfl_xor(lt2, 32);
    float pt = pd[mt] + __shfl_xor(pd[mt], 16);
    pt += __shfl_xor(pt, 32);
    if (g == 0) { st_m[wave][mt * 16 + n] = m[mt]; st_l[wave][mt * 16 + n] = lt2; st_p[wave][mt * 16 + n] = pt; }
  }
  __syncthreads();                                     // also: every wave is done with its tile region
  float* Ubuf = (float*)&vt[0][0];                     // [Hp][R]
  float f[MT];                                         // this wave's weight 2^(m_w - m*) per head
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int h = mt * 16 + n;
    const float ms = fmaxf(fmaxf(st_m[0][h], st_m[1][h]), fmaxf(st_m[2][h], st_m[3][h]));
    f[mt] = m[mt] > -INFINITY ? fast_exp2(m[mt] - ms) : 0.f;    // a wave without tiles adds nothing
  }
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    if (wave == w) {
      // U[i][j][mt][e] is (head 16 mt + n, column 32 i + 8 g + 2 e + j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < NKS; ++i) {
          float* dst = Ubuf + (size_t)(mt * 16 + n) * R + 32 * i + 8 * g;
          f32x4_t v0 = {U[i][0][mt][0], U[i][1][mt][0], U[i][0][mt][1], U[i][1][mt][1]};
          f32x4_t v1 = {U[i][0][mt][2], U[i][1][mt][2], U[i][0][mt][3], U[i][1][mt][3]};
          v0 *= f[mt];
          v1 *= f[mt];
          if (w > 0) { v0 += *(const f32x4_t*)dst; v1 += *(const f32x4_t*)(dst + 4); }
          *(f32x4_t*)dst = v0;
          *(f32x4_t*)(dst + 4) = v1;
        }
    }
    __syncthreads();
  }
  // ---- out: the split's sums and statistics, coalesced
  const size_t pb = ((size_t)b * S + su) * H;
  for (int i = threadIdx.x * 4; i < H * R; i += 256 * 4)
    *(f32x4_t*)(p.part_U + pb * R + i) = *(const f32x4_t*)(Ubuf + i);
  if ((int)threadIdx.x < H) {
    const int h = threadIdx.x;
    const float ms = fmaxf(fmaxf(st_m[0][h], st_m[1][h]), fmaxf(st_m[2][h], st_m[3][h]));
    float L = 0.f, pn = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float fw = st_m[w][h] > -INFINITY ? fast_exp2(st_m[w][h] - ms) : 0.f;
      L = fmaf(fw, st_l[w][h], L);
      pn = fmaf(fw, st_p[w][h], pn);
    }
    p.part_ml[(pb + h) * 2] = ms;
    p.part_ml[(pb + h) * 2 + 1] = L;
    if (p.defer_v && su == S - 1) p.pnew[(size_t)b * H + h] = pn;
  }
}

}  // namespace

bool attn_small_applies(int H, int r, int T, bool defer_v) {
  // 64 heads at rank 128 would not fit the register file (q' and U of all heads live in a wave)
  const int mt = (H + 15) / 16, nks = r / 32;
  return (r == 64 || r == 128) && H <= 64 && mt * nks <= 12 && (!defer_v || T >= 2);
}

ap_status launch_attn_small(ap_dtype dt, const uint16_t* Qp, const void* Ck, const void* Cv, float* part_ml,
                            float* part_U, float* pnew, float* scores, const int32_t* rank_k,
                            const int32_t* rank_v, const int32_t* bucket_off, const int32_t* bucket_idx, int F,
                            int B, int H, int T, int T_cap, int r, int nsplit, bool defer_v,
                            hipStream_t stream) {
  SmallParams p{Qp, (const uint16_t*)Ck, (const uint16_t*)Cv, part_ml, part_U, pnew, scores,
                B, T, T_cap, r, H, nsplit, B % 8 == 0 ? 1 : 0, defer_v ? 1 : 0,
                rank_k, rank_v, bucket_off, bucket_idx, F};
  const bool ragged = rank_k != nullptr || rank_v != nullptr;   // as everywhere in the library
  const int nb = B * nsplit;
  const int mt = (H + 15) / 16, nks = r / 32;
  hipEvent_t ev0, ev1;
  const bool timed = prof_events(&ev0, &ev1);          // the coefficient-streaming kernel of this call
#define AP_AS3(TAG, M, N, RG)                                                                          \
  do {                                                                                                 \
    if (timed) hipExtLaunchKernelGGL((attn_small<TAG, M, N, RG>), dim3(nb), dim3(256), 0, stream, ev0, ev1, 0u, p); \
    else hipLaunchKernelGGL((attn_small<TAG, M, N, RG>), dim3(nb), dim3(256), 0, stream, p);           \
  } while (0)
#define AP_AS2(TAG, M, N)                                                                              \
  do { if (ragged) AP_AS3(TAG, M, N, true); else AP_AS3(TAG, M, N, false); } while (0)
#define AP_AS1(TAG, M)                                                                                 \
  switch (nks) { case 2: AP_AS2(TAG, M, 2); break; default: AP_AS2(TAG, M, 4); break; }
#define AP_AS0(TAG)                                                                                    \
  switch (mt) { case 1: AP_AS1(TAG, 1) break; case 2: AP_AS1(TAG, 2) break; case 3: AP_AS1(TAG, 3) break; \
                default: AP_AS2(TAG, 4, 2); break; }          /* 64 heads: rank 64 only (see attn_small_applies) */
  if (dt == AP_F16) { AP_AS0(F16Tag) } else { AP_AS0(BF16Tag) }
#undef AP_AS0
#undef AP_AS1
#undef AP_AS2
#undef AP_AS3
  return AP_OK;
}

}  // namespace ap
