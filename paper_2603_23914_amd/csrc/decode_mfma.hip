// Decode attention over fp16 / bf16 coefficients on the matrix cores (gfx950).
//
// Paper Alg. 1 (partial decompression, scores, softmax, output) with the
// decompression matrices absorbed by associativity, so K and V are never rebuilt:
//   fold:    q'[h,j]  = sm_scale*log2(e) * sum_i Bk[j, h*d+i] q[h,i]      (basis_gemv.hip)
//   scores:  s[h,t]   = sum_{j<rk_t} Ck[t,j] q'[h,j]                       (kernel attn_partial)
//   softmax: online, base 2, fp32, per split of the token axis
//   sum:     u[h,j]   = sum_{t: rv_t>j} p[h,t] Cv[t,j]
//   merge:   splits combined with their (max, sum) pairs                   (basis_gemv.hip)
//   expand:  out[h,i] = sum_j u[h,j] Bv[j, h*d+i]
//
// attn_partial is the HBM-bound kernel.  One workgroup (8 waves) owns one (sequence, token
// split).  Coefficient tiles of 32 tokens travel HBM -> LDS with direct-to-LDS loads
// through a ring of 16-row units (K rows, K rows, V rows, V rows, ...), several units in
// flight while two are consumed, so no VGPR is spent on staging.  Every wave serves all
// heads on an eighth of the rank axis, so each tile byte is read from LDS exactly once:
//   S^T[t,h]  = Ck_tile[t,:] . q'^T      MFMA 16x16x32, A = tile rows (LDS), B = q' (VGPR);
//                                         the eight waves' partial sums meet in LDS and
//                                         each wave finalises the softmax of 1/8 of the heads
//   U^T[j,h] += Cv_tile^T[j,t] . P^T     MFMA 16x16x32, A = register transpose of the tile
//                                         (v_perm), B = P read back in operand layout
// For bf16 storage q' and P are split into hi+lo bf16 pairs (two MFMAs) so that the
// operand rounding stays far inside the 2e-3 tolerance; fp16 needs no split.
// int8 coefficients (one fp16 scale per token per 64 columns) travel as bytes and enter the
// MFMAs as exact fp16 integers; the scale is applied in fp32 (to the block's partial score, and
// folded into the softmax weight on the value side); everything else is the fp16 path.
#include "ap_common.hpp"
#include "mfma_ops.hpp"
#include <hip/hip_ext.h>

#include <cstdlib>

namespace ap {
namespace {

constexpr int kTile = 32;        // tokens per tile
constexpr int kHalf = 16;        // rows per LDS ring unit (half a tile of one matrix)
constexpr float kLazy = 8.0f;    // log2 slack before the softmax reference moves
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// The value rows are read once per launch: their direct-to-LDS loads carry the non-temporal hint
// (cache policy bit 1), so the stream does not displace what the caches hold for re-use (measured:
// 125.6 -> 121.3 us at the headline shape; the same hint on the key rows' register loads cost
// 13 us, so those stay plain).
constexpr int kStreamPolicy = 2;
__device__ __forceinline__ void dma16(const void* gsrc, void* lds_uniform) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_uniform, 16, 0, kStreamPolicy);
}

// s_waitcnt vmcnt(n) for a wave-uniform run-time n (the instruction takes an immediate).
#define AP_VMCNT_CASE(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
__device__ __forceinline__ void wait_vmcnt(int n) {
  switch (n) {
    AP_VMCNT_CASE(0) AP_VMCNT_CASE(1) AP_VMCNT_CASE(2) AP_VMCNT_CASE(3) AP_VMCNT_CASE(4)
    AP_VMCNT_CASE(5) AP_VMCNT_CASE(6) AP_VMCNT_CASE(7) AP_VMCNT_CASE(8) AP_VMCNT_CASE(9)
    AP_VMCNT_CASE(10) AP_VMCNT_CASE(11) AP_VMCNT_CASE(12) AP_VMCNT_CASE(13) AP_VMCNT_CASE(14)
    AP_VMCNT_CASE(15) AP_VMCNT_CASE(16) AP_VMCNT_CASE(17) AP_VMCNT_CASE(18) AP_VMCNT_CASE(19)
    AP_VMCNT_CASE(20) AP_VMCNT_CASE(21) AP_VMCNT_CASE(22) AP_VMCNT_CASE(23) AP_VMCNT_CASE(24)
    AP_VMCNT_CASE(25) AP_VMCNT_CASE(26) AP_VMCNT_CASE(27) AP_VMCNT_CASE(28) AP_VMCNT_CASE(29)
    AP_VMCNT_CASE(30) AP_VMCNT_CASE(31) AP_VMCNT_CASE(32) AP_VMCNT_CASE(33) AP_VMCNT_CASE(34)
    AP_VMCNT_CASE(35) AP_VMCNT_CASE(36) AP_VMCNT_CASE(37) AP_VMCNT_CASE(38) AP_VMCNT_CASE(39)
    AP_VMCNT_CASE(40) AP_VMCNT_CASE(41) AP_VMCNT_CASE(42)
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
  }
}
#undef AP_VMCNT_CASE

// Workgroup barrier that also orders this wave's LDS traffic, without the
// vmcnt(0) a full fence would add (direct-to-LDS loads must stay in flight).
__device__ __forceinline__ void wg_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <class Tag>
__device__ __forceinline__ void split_hi_lo(float x, uint16_t& hi, uint16_t& lo) {
  hi = f32_to_bits(x, Tag{});
  lo = f32_to_bits(x - bits_to_f32(hi, Tag{}), Tag{});
}


// int8 codes -> the same integers as fp16 values, two at a time, exactly.  A byte b (two's
// complement) xor 0x80 is b+128 as an unsigned byte u; the fp16 bit pattern 0x6400|u is exactly
// 1024+u, so subtracting 1152 leaves b.  The matrix cores multiply these integer-valued operands
// (products and fp32 sums of a 64-column block are exact), and the block's fp16 scale is applied
// in fp32 afterwards: a coefficient's value is code * fp32(scale), never rounded on its own.
typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t code2(uint32_t biased /* 0x64uu64uu */) {
  const h2_t off = {(_Float16)-1152.0f, (_Float16)-1152.0f};
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, biased) + off);
}
// 8 consecutive codes of one row (two dwords) -> MFMA operand (8 fp16 integers)
__device__ __forceinline__ u32x4_t code_row8(uint32_t c0, uint32_t c1) {
  const uint32_t k = 0x64646464u;
  const uint32_t x0 = c0 ^ 0x80808080u, x1 = c1 ^ 0x80808080u;
  u32x4_t o;
  o[0] = code2(__builtin_amdgcn_perm(k, x0, 0x04010400u));
  o[1] = code2(__builtin_amdgcn_perm(k, x0, 0x04030402u));
  o[2] = code2(__builtin_amdgcn_perm(k, x1, 0x04010400u));
  o[3] = code2(__builtin_amdgcn_perm(k, x1, 0x04030402u));
  return o;
}

// 4-bit codes (two per byte, each nibble the code plus 8): a dword holds eight codes, nibble j
// column c0 + j.  0x6400 | u is 1024 + u in fp16, so subtracting 1032 leaves the code exactly.
__device__ __forceinline__ uint32_t code2_4(uint32_t biased /* 0x640u640u */) {
  const h2_t off = {(_Float16)-1032.0f, (_Float16)-1032.0f};
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, biased) + off);
}
// eight codes of one row (one dword) -> MFMA operand; operand slots (2k, 2k+1) hold columns
// (k, k+4) of the eight, so the other operand is loaded in that column order
__device__ __forceinline__ u32x4_t code_row8_i4(uint32_t d) {
  u32x4_t o;
#pragma unroll
  for (int k = 0; k < 4; ++k) o[k] = code2_4(((d >> (4 * k)) & 0x000f000fu) | 0x64006400u);
  return o;
}

// ------------------------------------------------------------------------------------------
// tile kernels (unrolled to the compile-time maximum, left early on the run-time count)
// ------------------------------------------------------------------------------------------
// Partial scores of one 32-token tile over this wave's score k-steps (32 columns each), for
// all MT head tiles.  A[i][tt]: rows 16tt..16tt+15 of the tile at k-step i, in registers.
// k-steps this wave does not own hold zero rows and zero q' (no branch: the accumulators
// stay in one straight-line live range).
// nlive: k-steps of this wave that lie below the tile's key rank (wave-uniform; the others hold
// zero rows and are skipped: at a quarter of the rank a tile costs a quarter of the products).
template <class Tag, int MT, bool SPLIT, int NKW>
__device__ __forceinline__ void score_tile(const u32x4_t (&A)[NKW][2],
                                           const u32x4_t (&qhi)[NKW][MT],
                                           const u32x4_t (&qlo)[SPLIT ? NKW : 1][MT],
                                           f32x4_t (&s)[MT][2], int nlive = NKW) {
#pragma unroll
  for (int i = 0; i < NKW; ++i) {
    if (i >= nlive) break;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      s[mt][0] = Mfma<Tag>::run(A[i][0], qhi[i][mt], s[mt][0]);
      s[mt][1] = Mfma<Tag>::run(A[i][1], qhi[i][mt], s[mt][1]);
    }
    if (SPLIT) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        s[mt][0] = Mfma<Tag>::run(A[i][0], qlo[i][mt], s[mt][0]);
        s[mt][1] = Mfma<Tag>::run(A[i][1], qlo[i][mt], s[mt][1]);
      }
    }
  }
}

// Weighted coefficient sum of one tile over all 128-column groups (256 bytes apart).  In
// each group the wave owns four 16-byte chunks (32 columns): MFMA row m = 4g'+e reads dword
// e of chunk g', so the 16 lanes of a row group read 64 contiguous bytes and the four row
// groups fall on different banks (no LDS bank conflicts).  vA / vB: rows 0-15 / 16-31 of
// the tile, already offset to this lane's dword.
template <class Tag, int MT, bool SPLIT, int NGL>
__device__ __forceinline__ void wsum_tile(const char* vA, const char* vB, int pitch,
                                          int cols_left, int n, const u32x4_t (&Phi)[MT],
                                          const u32x4_t (&Plo)[MT], const float (&alpha)[MT],
                                          f32x4_t (&U)[NGL][2][MT]) {
  // lanes whose columns lie at or beyond the rank contribute zeros (no branch around the
  // MFMAs: the accumulators stay in one straight-line live range); the rows of group i+1
  // are fetched while group i is multiplied
  // alpha is 1 except when a head's softmax reference exponent moved (rare: the reference
  // follows the maximum lazily), so the rescaling of the sums is skipped wave-wide otherwise
  {
    bool moved = false;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) moved |= alpha[mt] != 1.0f;
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
      for (int i = 0; i < NGL; ++i)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) { U[i][0][mt] *= alpha[mt]; U[i][1][mt] *= alpha[mt]; }
    }
  }
  uint32_t nx[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (n * 2 < cols_left) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      nx[e] = *(const uint32_t*)(vA + e * pitch);
      nx[4 + e] = *(const uint32_t*)(vB + e * pitch);
    }
  }
#pragma unroll
  for (int i = 0; i < NGL; ++i) {
    if (i * 128 >= cols_left) break;         // wave-uniform: the group lies beyond the value rank
    uint32_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { v[e] = nx[e]; nx[e] = 0; }
    if (i + 1 < NGL && (i + 1) * 128 + n * 2 < cols_left) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        nx[e] = *(const uint32_t*)(vA + e * pitch + (i + 1) * 256);
        nx[4 + e] = *(const uint32_t*)(vB + e * pitch + (i + 1) * 256);
      }
    }
    // 8x2 transpose of 16-bit elements: operand j holds one column of the 8 tokens
    u32x4_t te, to;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      te[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], 0x05040100u);
      to[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], 0x07060302u);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      U[i][0][mt] = Mfma<Tag>::run(te, Phi[mt], U[i][0][mt]);
      U[i][1][mt] = Mfma<Tag>::run(to, Phi[mt], U[i][1][mt]);
    }
    if (SPLIT) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        U[i][0][mt] = Mfma<Tag>::run(te, Plo[mt], U[i][0][mt]);
        U[i][1][mt] = Mfma<Tag>::run(to, Plo[mt], U[i][1][mt]);
      }
    }
  }
}

// int8 variant of score_tile.  A wave owns 64-column scale blocks w, w+4, ...; per block and
// 16-row half it holds the lane's 16 codes (columns 64m + 16g .. +15 of its row) and the
// scale of its row (token 16 tt + n).  Codes 0-7 feed one MFMA and codes 8-15 the next (q' is
// loaded with the same column order), so a block is two k-steps.  The block's sum over the
// integer codes is exact in fp32; it is multiplied by the token's scale in fp32 and added to the
// scores.  A lane's results belong to tokens 16 tt + 4 g + e, whose scales sit in lanes 4 g + e.
// 4-bit codes (I4): the lane's 16 codes of a block are two dwords, one per k-step.
template <int MT, int NBW, bool I4>
__device__ __forceinline__ void score_tile_i8(const u32x4_t (&Araw)[NBW][2],
                                              const uint32_t (&ksc)[NBW][2], int g,
                                              const u32x4_t (&qhi)[2 * NBW][MT],
                                              f32x4_t (&s)[MT][2]) {
#pragma unroll
  for (int i = 0; i < NBW; ++i) {
    u32x4_t a0[2], a1[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      a0[tt] = I4 ? code_row8_i4(Araw[i][tt][0]) : code_row8(Araw[i][tt][0], Araw[i][tt][1]);
      a1[tt] = I4 ? code_row8_i4(Araw[i][tt][1]) : code_row8(Araw[i][tt][2], Araw[i][tt][3]);
    }
    f32x4_t pb[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
      pb[mt][0] = Mfma<F16Tag>::run(a0[0], qhi[2 * i][mt], z);
      pb[mt][1] = Mfma<F16Tag>::run(a0[1], qhi[2 * i][mt], z);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      pb[mt][0] = Mfma<F16Tag>::run(a1[0], qhi[2 * i + 1][mt], pb[mt][0]);
      pb[mt][1] = Mfma<F16Tag>::run(a1[1], qhi[2 * i + 1][mt], pb[mt][1]);
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t sb = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * (4 * g + e), (int)ksc[i][tt]);
        const float sc = bits_to_f32((uint16_t)sb, F16Tag{});
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) s[mt][tt][e] = fmaf(sc, pb[mt][tt][e], s[mt][tt][e]);
      }
  }
}

// int8 variant of wsum_tile.  Column groups are 256 wide; in each the wave owns 64 bytes (one
// scale block).  Lane (n, g) reads dword n of those bytes for its 8 tokens: four codes, i.e.
// columns 4n .. 4n+3 of the wave's 64, one MFMA per byte position.  vs: this tile's value
// scales in LDS as [scale block][32 tokens] fp16.
// The codes enter the product as exact integers; a token's scale for the block is folded into
// its softmax weight in fp32 (P32: the lane's eight weights per head tile, tokens 4g .. 4g+3
// and 16+4g .. +3), and that product is rounded to fp16 once.
template <int MT, int NGL>
__device__ __forceinline__ void wsum_tile_i8(const char* vA, const char* vB, int pitch, int r,
                                             int cp, int g, const uint16_t* vs,
                                             const f32x4_t (&P32)[MT][2], const float (&alpha)[MT],
                                             f32x4_t (&U)[NGL][4][MT]) {
  // alpha is 1 except when a head's softmax reference exponent moved (rare): the rescaling of
  // the sums is skipped wave-wide otherwise, as in wsum_tile
  {
    bool moved = false;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) moved |= alpha[mt] != 1.0f;
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
      for (int i = 0; i < NGL; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) U[i][j][mt] *= alpha[mt];
    }
  }
#pragma unroll
  for (int i = 0; i < NGL; ++i) {
    const int blk = 4 * i + cp;
    uint32_t v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    u32x2_t s01 = {0, 0}, s23 = {0, 0};
    if (blk * 64 < r) {                       // wave-uniform: the block exists at this rank
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] = *(const uint32_t*)(vA + e * pitch + i * 256);
        v[4 + e] = *(const uint32_t*)(vB + e * pitch + i * 256);
      }
      s01 = *(const u32x2_t*)(vs + blk * kTile + 4 * g);          // tokens 4g .. 4g+3
      s23 = *(const u32x2_t*)(vs + blk * kTile + 16 + 4 * g);     // tokens 16+4g .. +3
    }
    const uint32_t sc[4] = {s01[0], s01[1], s23[0], s23[1]};
    u32x4_t Psc[MT];                           // weight * scale of this block, per head tile
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float f0 = lo_to_f32(sc[k], F16Tag{}), f1 = hi_to_f32(sc[k], F16Tag{});
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        Psc[mt][k] = cvt_pack(P32[mt][k >> 1][2 * (k & 1)] * f0, P32[mt][k >> 1][2 * (k & 1) + 1] * f1, F16Tag{});
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // byte j of two tokens -> low bytes of the two halves, then bias into 0x64uu
      const uint32_t sel = 0x0c000c00u | ((uint32_t)(4 + j) << 16) | (uint32_t)j;
      u32x4_t op;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        op[k] = code2(__builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], sel) ^ 0x64806480u);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        U[i][j][mt] = Mfma<F16Tag>::run(op, Psc[mt], U[i][j][mt]);
    }
  }
}

// 4-bit variant.  The wave owns the 64-column scale blocks cp, cp + 4, ... (32 bytes of a row
// each).  A block's eight dwords feed sixteen MFMA rows: row n reads dword n & 7 and takes the
// nibbles 4 (n >> 3) + j, j = 0..3, one MFMA per j; row n is then column 8 (n & 7) + 4 (n >> 3) + j
// of the block, so all sixteen rows of a product share one scale block and the token's scale can
// be folded into its weight as for int8.  vA / vB: rows 0-15 / 16-31 of the tile, offset to the
// lane's token rows only.
template <int MT, int NGL>
__device__ __forceinline__ void wsum_tile_i4(const char* vA, const char* vB, int pitch, int r,
                                             int cp, int n, int g, const uint16_t* vs,
                                             const f32x4_t (&P32)[MT][2], const float (&alpha)[MT],
                                             f32x4_t (&U)[NGL][4][MT]) {
  const int doff = (n & 7) * 4;              // this row's dword inside a block
  const int sh0 = 16 * (n >> 3);             // its first nibble
  {                                          // rescale only when a reference exponent moved (rare)
    bool moved = false;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) moved |= alpha[mt] != 1.0f;
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
      for (int i = 0; i < NGL; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) U[i][j][mt] *= alpha[mt];
    }
  }
#pragma unroll
  for (int i = 0; i < NGL; ++i) {
    {
      const int blk = 4 * i + cp;
      uint32_t v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      u32x2_t s01 = {0, 0}, s23 = {0, 0};
      if (blk * 64 < r) {                     // wave-uniform: the block exists at this rank
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = *(const uint32_t*)(vA + e * pitch + blk * 32 + doff);
          v[4 + e] = *(const uint32_t*)(vB + e * pitch + blk * 32 + doff);
        }
        s01 = *(const u32x2_t*)(vs + blk * kTile + 4 * g);
        s23 = *(const u32x2_t*)(vs + blk * kTile + 16 + 4 * g);
      }
      const uint32_t sc[4] = {s01[0], s01[1], s23[0], s23[1]};
      u32x4_t Psc[MT];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float f0 = lo_to_f32(sc[k], F16Tag{}), f1 = hi_to_f32(sc[k], F16Tag{});
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          Psc[mt][k] = cvt_pack(P32[mt][k >> 1][2 * (k & 1)] * f0, P32[mt][k >> 1][2 * (k & 1) + 1] * f1, F16Tag{});
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int sh = sh0 + 4 * j;
        u32x4_t op;
#pragma unroll
        for (int k = 0; k < 4; ++k)
          op[k] = code2_4(((v[2 * k] >> sh) & 0xfu) | (((v[2 * k + 1] >> sh) & 0xfu) << 16) | 0x64006400u);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          U[i][j][mt] = Mfma<F16Tag>::run(op, Psc[mt], U[i][j][mt]);
      }
    }
  }
}

// Butterfly steps inside groups of 8 lanes with DPP (VALU speed, no LDS crossbar):
// xor 1 and xor 2 as quad permutes; the third step mirrors each half-row, which pairs the
// two quads of an 8-lane group (all lanes of a quad already agree after the first two).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  const int v = __builtin_bit_cast(int, x);
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float max8(float x) {
  x = fmaxf(x, dpp_f32<0xB1>(x));    // quad_perm [1,0,3,2]
  x = fmaxf(x, dpp_f32<0x4E>(x));    // quad_perm [2,3,0,1]
  x = fmaxf(x, dpp_f32<0x141>(x));   // row_half_mirror
  return x;
}
__device__ __forceinline__ float sum8(float x) {
  x += dpp_f32<0xB1>(x);
  x += dpp_f32<0x4E>(x);
  x += dpp_f32<0x141>(x);
  return x;
}

// A non-inlined device function receives its arguments in VGPRs, so the compiler treats
// everything derived from them as divergent.  These put wave-uniform values back into SGPRs.
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
template <class P>
__device__ __forceinline__ P* uni_ptr(P* ptr) {
  const uint64_t v = (uint64_t)ptr;
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
  return (P*)(((uint64_t)hi << 32) | lo);
}

// ------------------------------------------------------------------------------------------
// attn_partial
// ------------------------------------------------------------------------------------------
struct AttnParams {
  const uint16_t* Qp;   // [B][2][Hp][r]
  const uint16_t* Ck;   // [B][T_cap][r]
  const uint16_t* Cv;
  const uint16_t* Sk;   // int8 / 4-bit coefficients only: fp16 scales [B][T_cap][r/64]
  const uint16_t* Sv;
  int qbits;            // 8 or 4 when Sk is given
  float* part_ml;       // [B][S][H][2]   (softmax reference exponent in log2 units, sum)
  float* part_U;        // [B][S][H][r]
  int B, T, T_cap, r, H, nsplit;
  int xcd_aware;        // workgroup numbering, see wg_coords
  int nh;               // C_v LDS ring depth in 16-row units (even, >= 2)
  // rank-ragged launches only: the group lists of ap_select_ranks and the per-token ranks
  const int32_t* rank_k;      // [B][T] or null (= r)
  const int32_t* rank_v;
  const int32_t* bucket_off;  // [B][F+1]
  const int32_t* bucket_idx;  // [B][T]
  int F;
  int ntl_cap;          // most tiles a split can own (sizes the LDS index table)
  // fused decode step: the newest token (row T-1) is scored like every other, but its value
  // row does not exist yet; its softmax weight is exported and the expansion pass adds it
  int defer_v;          // 0 or 1
  float* pnew;          // [B][H] weight of token T-1 relative to the reference of the split that holds it
  int* pnew_split;      // [B] ... and which split that is
  float* scores;        // [B][T_cap][H] scaled logits in natural-log units, or null
  int dbg;              // kernel studies (AP_KERNEL_TIMERS builds only, else 0): 1 = no loads,
                        // 2 = no math, 4 = phase timers, 8 = per-tile stamps
  unsigned long long* dbg_out;
};

// Eight waves (two per SIMD) in two roles, every one serving ALL heads (MT tiles of 16)
// on a quarter of the rank axis:
//   score waves 0-3:  k-steps w, w+4, ... of S^T = Ck_tile . q'^T.  They hold q' and fetch
//                     their slice of the C_k rows straight from global memory into MFMA
//                     operand registers (16 rows x 64 B per load instruction), one tile
//                     ahead; their four partial score tiles meet in LDS.
//   sum waves 4-7:    32 of every 128 columns of U^T += Cv_tile^T . P^T.  They hold U and
//                     stream the C_v rows HBM -> LDS with direct-to-LDS loads through a ring
//                     of 16-row units, several tiles ahead, so no VGPR is spent on staging
//                     and every LDS byte is read exactly once.
//   all eight waves:  finalise the softmax of 2*MT heads each (eight lanes per head): they
//                     keep (reference exponent, sum) and publish the weights in MFMA operand
//                     layout plus a per-head rescale factor.
// The score waves work on tile t+1 while the sum waves accumulate tile t; two workgroup
// barriers per tile ("partial scores ready", "weights ready") keep them in step.  The two
// roles are separate non-inlined functions (same barrier sequence), so q' and U never
// compete for registers.  The softmax reference exponent only moves when a score exceeds
// it by more than kLazy, so the rescale factor is 1 on almost every tile.
//
// Workgroup id -> (sequence, split).  Consecutive workgroup ids go to different XCDs (8 of
// them, each with its own L2).  With whole groups of 8 sequences (xcd_aware), sequence b lives
// on XCD b % 8 and its splits are neighbours in that XCD's dispatch order: the folded query of
// a sequence is fetched from HBM once and found in L2 by the other splits.  Smaller batches
// keep the plain numbering, which spreads a sequence's splits over all XCDs.
__device__ __forceinline__ void wg_coords(int nsplit, int xcd_aware, int& b, int& s) {
  const int id = __builtin_amdgcn_readfirstlane((int)blockIdx.x);
  if (xcd_aware) {
    const int k = id >> 3;
    b = (k / nsplit) * 8 + (id & 7);
    s = k - (k / nsplit) * nsplit;
  } else {
    b = id / nsplit;
    s = id - b * nsplit;
  }
}

// State every wave carries through the token loop, whatever its role.
// Rank-ragged launches (RAGGED): a tile is 32 tokens of ONE rank group, taken from the
// group's index list, so the rank is uniform inside a tile and nothing diverges; tiles are
// dealt to the splits round-robin (tile s, s + nsplit, ...), which gives every split the
// same mix of ranks.  Each workgroup first copies the token indices of its tiles and each
// tile's (token count, key rank, value rank) into LDS; the row loads then gather through
// that table.  Columns at or beyond a tile's rank are neither fetched from HBM (their loads
// are redirected to bytes the wave fetches anyway) nor allowed into the products.
// Token-split mode (TS, ranks up to 128): the four score waves each own every fourth TILE and
// all of the rank axis, instead of a quarter of the rank axis of every tile.  A score wave's
// tile is then complete without the other waves' partial sums, and one pair of barriers covers
// four tiles: at small ranks the tile loop is bound by that dependency chain, not by memory.
// Q: coefficient storage, 0 = 16-bit, 1 = int8 codes, 2 = 4-bit codes (both with fp16 scales).
template <class Tag, int MT, bool SPLIT, bool RAGGED, int Q, bool TS = false>
struct WaveCtx {
  static constexpr bool I8 = Q != 0, I4 = Q == 2;
  static constexpr int NSUB = TS ? 4 : 1;   // tiles per barrier pair
  static constexpr int HPW = 2 * MT;     // heads finalised per wave
  // bytes of a coefficient row
  static __device__ __forceinline__ int row_bytes_of(int r) { return I4 ? r >> 1 : (I8 ? r : 2 * r); }

  int w, lane, n, g, b, s;
  int r, T, H, nh, nsplit, dbg;
  int pitch, nblk, unit_bytes;
  char* ring;
  f32x4_t* xchg;     // [4 score waves][16*MT heads][9]: 8 slots (4*tt+g) + 1 pad per head
  u32x4_t* Pbuf;     // [MT][hi,lo][64 lanes]
  float* abuf;       // [16*MT] rescale factors
  uint16_t* vsb;     // I8: [2][r/64][32] value scales of the tile in flight (fp16 bits)
  int* idxb;         // RAGGED: [ntl][32] token index of every tile slot (tail slots repeat the last)
  int* meta;         // RAGGED: [ntl][4] = tokens in the tile, key rank, value rank, 1 + slot of the
                     // deferred newest token (0: not in this tile)
  uint32_t row_bytes;
  int t_lo, ntl;     // first tile (token-split mode) and number of tiles of this split
  int tok_a, tok_h, tok_rem;   // contiguous tiles: the split's first token; its first tok_rem tiles
                               // hold tok_h + 1 tokens, the others tok_h
  int Tv;            // value rows that exist: T, or T-1 while the newest token's row is deferred
  float* pnew;
  int* pnew_split;
  float* scores;     // this sequence's [T_cap][H] logits, or null
  int T_cap;
  // softmax ownership: lane = 8*head_local + slot, slot = 4*tt + gg covers tokens
  // 16*tt + 4*gg .. +3 of the tile for head o_hh
  bool owner;
  int o_hh, o_tt, o_gg, o_mt, o_lane;
  float m_ref, l_part;

  __device__ __forceinline__ void init(const AttnParams& p) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x;
    w = __builtin_amdgcn_readfirstlane(tid >> 6);
    lane = tid & 63; n = lane & 15; g = lane >> 4;
    r = uni(p.r); T = uni(p.T); H = uni(p.H); nh = uni(p.nh); nsplit = uni(p.nsplit); dbg = uni(p.dbg);
    wg_coords(nsplit, uni(p.xcd_aware), b, s);
    Tv = T - uni(p.defer_v);
    pnew = uni_ptr(p.pnew);
    pnew_split = uni_ptr(p.pnew_split);
    T_cap = uni(p.T_cap);
    scores = uni_ptr(p.scores);
    if (scores) scores += (size_t)b * H * T_cap;
    // ring unit geometry: 16 rows of (cpr+1) 16-byte chunks (one pad chunk per row shifts
    // consecutive rows across the LDS banks)
    const int cpr = row_bytes_of(r) >> 4;
    pitch = (cpr + 1) * 16;
    nblk = (kHalf * (cpr + 1) + 63) >> 6;
    unit_bytes = nblk * 1024;
    ring = smem;
    xchg = (f32x4_t*)(smem + nh * unit_bytes);
    Pbuf = (u32x4_t*)(xchg + 4 * 16 * MT * 9);
    abuf = (float*)(Pbuf + NSUB * MT * 2 * 64);
    row_bytes = (uint32_t)row_bytes_of(r);
    vsb = (uint16_t*)(abuf + NSUB * 16 * MT);
    tok_a = 0; tok_h = kTile; tok_rem = 0;
    if (!RAGGED && TS) {
      const int ntiles = (T + kTile - 1) / kTile;
      t_lo = (int)(((int64_t)s * ntiles) / nsplit);
      ntl = (int)(((int64_t)(s + 1) * ntiles) / nsplit) - t_lo;
    } else if (!RAGGED) {
      // The splits share the TOKENS evenly, not the 32-token tiles: a split of n tokens walks
      // ceil(n / 32) tiles of floor(n / tiles) or one more tokens each.  A tile still fetches the
      // 32 consecutive rows from its first token on; the rows beyond its own count belong to the
      // next tile, are masked here and come out of L2 there.  With whole tiles dealt out instead,
      // one split of a sequence owns a tile more than the others whenever the tile count is not a
      // multiple of the split count (34 against 33 at T = 4240 in four splits).  The launch takes
      // as long as before (a tile costs the same whether 31 or 32 of its rows count, and the
      // longest split still walks 34), but every split now does the same work at any T.
      t_lo = 0;
      tok_a = (int)(((int64_t)s * T) / nsplit);
      const int n_tok = (int)(((int64_t)(s + 1) * T) / nsplit) - tok_a;
      ntl = (n_tok + kTile - 1) / kTile;
      tok_h = ntl > 0 ? n_tok / ntl : 0;
      tok_rem = n_tok - tok_h * ntl;
    } else {
      idxb = (int*)(vsb + (I8 ? 2 * (r >> 6) * kTile : 0));
      meta = idxb + uni(p.ntl_cap) * kTile;
      build_tile_table(p);
    }
    owner = lane < 8 * HPW;
    o_hh = w * HPW + (lane >> 3);
    o_tt = (lane >> 2) & 1; o_gg = lane & 3;
    o_mt = o_hh >> 4; o_lane = (o_hh & 15) + 16 * o_gg;
    m_ref = -INFINITY; l_part = 0.f;
  }

  // RAGGED: tiles of this split, their token indices and ranks into LDS (all 512 threads).
  __device__ __forceinline__ void build_tile_table(const AttnParams& p) {
    const int F = uni(p.F);
    const int32_t* boff = uni_ptr(p.bucket_off) + (size_t)b * (F + 1);
    const int32_t* bidx = uni_ptr(p.bucket_idx) + (size_t)b * T;
    const int32_t* rk_arr = uni_ptr(p.rank_k);
    const int32_t* rv_arr = uni_ptr(p.rank_v);
    int off[9], ts[9];                     // group g: list positions off[g]..off[g+1], first tile ts[g]
    off[0] = boff[0];
    ts[0] = 0;
#pragma unroll
    for (int g2 = 0; g2 < 8; ++g2) {
      off[g2 + 1] = g2 < F ? boff[g2 + 1] : off[g2];
      int c = off[g2 + 1] - off[g2];
      c = c < 0 ? 0 : c;
      ts[g2 + 1] = ts[g2] + ((c + kTile - 1) >> 5);
    }
    const int ntot = ts[8];
    t_lo = 0;
    ntl = s < ntot ? (ntot - s + nsplit - 1) / nsplit : 0;
    const int cap = uni(p.ntl_cap);
    ntl = ntl < cap ? ntl : cap;           // never beyond the table (host sizes it for the worst case)
    // Visiting order: the split's tiles come in group order (high ranks first); walked with a
    // stride of about ntl / F (coprime to ntl) high- and low-rank tiles alternate, so that the
    // short tiles' products run while the long tiles' rows are still on their way.
    int stride = ntl / (F > 0 ? F : 1);
    stride = stride < 1 ? 1 : stride;
    for (;; ++stride) {
      int x = stride, y = ntl;
      while (y) { const int tmp = x % y; x = y; y = tmp; }
      if (x == 1 || ntl <= 1) break;
    }
    for (int e = threadIdx.x; e < ntl * kTile; e += 512) {
      const int i = e >> 5, l = e & 31;
      const int isrc = ntl > 1 ? (int)(((int64_t)i * stride) % ntl) : 0;
      const int j = s + isrc * nsplit;
      int o0 = off[0], o1 = off[1], t0 = 0;
#pragma unroll
      for (int k = 1; k < 8; ++k)
        if (k < F && j >= ts[k]) { o0 = off[k]; o1 = off[k + 1]; t0 = ts[k]; }
      const int pos0 = o0 + (j - t0) * kTile;
      int cnt = o1 - pos0;
      cnt = cnt > kTile ? kTile : cnt;
      int pos = pos0 + (l < cnt ? l : cnt - 1);
      pos = pos < 0 ? 0 : (pos < T ? pos : T - 1);
      int tok = bidx[pos];
      tok = tok < 0 ? 0 : (tok < T ? tok : T - 1);
      idxb[e] = tok;
      // the 32 slots of a tile are 32 consecutive lanes: the slot of the deferred newest token
      const unsigned long long hit = __ballot(Tv != T && tok == T - 1 && l < cnt);
      const uint32_t hit32 = (uint32_t)((lane & 32) ? hit >> 32 : hit);
      if (l == 0) {
        int rk = rk_arr ? rk_arr[(size_t)b * T + tok] : r;
        int rv = rv_arr ? rv_arr[(size_t)b * T + tok] : r;
        rk = rk < 0 ? 0 : (rk < r ? rk : r);
        rv = rv < 0 ? 0 : (rv < r ? rv : r);
        meta[4 * i + 0] = cnt;
        meta[4 * i + 1] = rk;
        meta[4 * i + 2] = rv;
        meta[4 * i + 3] = hit32 ? __ffs((int)hit32) : 0;
      }
    }
    wg_barrier();
  }

  // First token of local tile t (contiguous tiles).
  __device__ __forceinline__ int tok0(int t) const {
    if (TS) return (t_lo + t) * kTile;
    return tok_a + t * tok_h + (t < tok_rem ? t : tok_rem);
  }

  // Tokens of local tile t that count (the rest of the 32 slots is masked out of the softmax).
  __device__ __forceinline__ int tile_valid(int t) const {
    if (TS && t >= ntl) return 0;        // a slot of the last round without a tile
    if (RAGGED) return uni(meta[4 * t]);
    if (!TS) return tok_h + (t < tok_rem ? 1 : 0);
    const int left = T - tok0(t);
    return left < kTile ? left : kTile;
  }

  // Slot of the deferred newest token in local tile t, or -1 when it is not one of its tokens.
  __device__ __forceinline__ int tile_new(int t) const {
    if (Tv == T || (TS && t >= ntl)) return -1;
    if (RAGGED) return uni(meta[4 * t + 3]) - 1;
    const int nl = T - 1 - tok0(t);
    return nl < tile_valid(t) ? nl : -1;
  }

  // Softmax of this wave's heads for a tile whose first `valid` slots hold tokens (after
  // the score waves' partial tiles are in xchg).  newl: slot of the deferred token, if any:
  // its weight counts in the sum, is exported, and stays out of the value products.
  // sub: which of the NSUB tiles of this barrier pair (its scores sit in slot `sub` of xchg,
  // its weights go to slot `sub` of Pbuf / abuf).
  __device__ __forceinline__ void finalize_softmax(int valid, int newl, int t, int sub = 0) {
    if (!owner) return;
    const int xi = o_hh * 9 + (lane & 7);
    f32x4_t sc;
    if (TS) {
      sc = xchg[sub * 16 * MT * 9 + xi];          // complete: one wave scored the whole rank axis
    } else {
      sc = xchg[xi];
#pragma unroll
      for (int sw = 1; sw < 4; ++sw) sc += xchg[sw * 16 * MT * 9 + xi];
    }
    if (scores && o_hh < H) {                   // logits out, for importance tracking: [token][head]
      const int slot = 16 * o_tt + 4 * o_gg;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (slot + i < valid) {
          const int tok = RAGGED ? idxb[t * kTile + slot + i] : tok0(t) + slot + i;
          scores[(size_t)tok * H + o_hh] = sc[i] * kLn2;
        }
      }
    }
    if (valid < kTile) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (16 * o_tt + 4 * o_gg + i >= valid) sc[i] = -INFINITY;
    }
    float tmax = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
    tmax = max8(tmax);
    float alpha = 1.0f;
    if (tmax > m_ref + kLazy) {                 // same decision in the 8 lanes of a head
      const float m_upd = fmaxf(m_ref, tmax);   // finite: every tile holds a valid token
      alpha = fast_exp2(m_ref - m_upd);
      m_ref = m_upd;
      l_part *= alpha;
    }
    float p0 = fast_exp2(sc[0] - m_ref), p1 = fast_exp2(sc[1] - m_ref);
    float p2 = fast_exp2(sc[2] - m_ref), p3 = fast_exp2(sc[3] - m_ref);
    float pdef = 0.f;
    if (newl >= 0 && newl < kTile) {            // wave-uniform: this tile holds the deferred token
      const int li = newl - (16 * o_tt + 4 * o_gg);
      if (li == 0) { pdef = p0; p0 = 0.f; }
      if (li == 1) { pdef = p1; p1 = 0.f; }
      if (li == 2) { pdef = p2; p2 = 0.f; }
      if (li == 3) { pdef = p3; p3 = 0.f; }
      if (li >= 0 && li < 4 && o_hh < H) {
        pnew[(size_t)b * H + o_hh] = pdef;
        if (o_hh == 0) pnew_split[b] = s;
      }
    }
    u32x2_t hi, lo = {0, 0};
    hi[0] = cvt_pack(p0, p1, Tag{});
    hi[1] = cvt_pack(p2, p3, Tag{});
    float k0 = lo_to_f32(hi[0], Tag{}), k1 = hi_to_f32(hi[0], Tag{});
    float k2 = lo_to_f32(hi[1], Tag{}), k3 = hi_to_f32(hi[1], Tag{});
    if (SPLIT) {
      lo[0] = cvt_pack(p0 - k0, p1 - k1, Tag{});
      lo[1] = cvt_pack(p2 - k2, p3 - k3, Tag{});
      k0 += lo_to_f32(lo[0], Tag{});
      k1 += hi_to_f32(lo[0], Tag{});
      k2 += lo_to_f32(lo[1], Tag{});
      k3 += hi_to_f32(lo[1], Tag{});
    }
    if (I8) {
      // int8 coefficients: the weights stay fp32 (the sum waves fold the value scales in before
      // rounding); the two 16-byte slots of a lane hold tokens 4g .. 4g+3 and 16+4g .. +3
      l_part += (p0 + p1) + (p2 + p3);
      const f32x4_t pv = {p0, p1, p2, p3};
      *(f32x4_t*)(Pbuf + ((sub * MT + o_mt) * 2 + o_tt) * 64 + o_lane) = pv;
      if ((lane & 7) == 0) abuf[sub * 16 * MT + o_hh] = alpha;
      return;
    }
    l_part += (k0 + k1) + (k2 + k3) + pdef;     // the sum uses the values the MFMA will see
    // weights in B-operand layout: lane (n, g) of head tile mt holds tokens 4g..4g+3
    // (dwords 0,1) and 16+4g..+3 (dwords 2,3)
    u32x2_t* ph = (u32x2_t*)(Pbuf + ((sub * MT + o_mt) * 2 + 0) * 64 + o_lane) + o_tt;
    *ph = hi;
    if (SPLIT) *(ph + 2 * 64) = lo;             // [sub][o_mt][1][o_lane]
    if ((lane & 7) == 0) abuf[sub * 16 * MT + o_hh] = alpha;
  }

  // Token-split mode: the softmax of the four tiles t0 .. t0+3 of a round in one go (one
  // maximum, one move of the reference exponent, sixteen independent exponentials per lane)
  // instead of four dependent passes.  The rescale factor goes with the first tile; the
  // other three carry 1.
  __device__ __forceinline__ void finalize_softmax4(int t0) {
    if (!owner) return;
    const int xi = o_hh * 9 + (lane & 7);
    const int slot = 16 * o_tt + 4 * o_gg;       // this lane's first token slot in a tile
    f32x4_t sc[4];
    int valid[4], newl[4];
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      sc[sub] = xchg[sub * 16 * MT * 9 + xi];
      valid[sub] = tile_valid(t0 + sub);
      newl[sub] = tile_new(t0 + sub);
    }
    if (scores && o_hh < H) {                   // logits out, for importance tracking: [token][head]
#pragma unroll
      for (int sub = 0; sub < 4; ++sub)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (slot + i < valid[sub])
            scores[(size_t)(tok0(t0 + sub) + slot + i) * H + o_hh] = sc[sub][i] * kLn2;
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 4; ++sub)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (slot + i >= valid[sub]) sc[sub][i] = -INFINITY;
        tmax = fmaxf(tmax, sc[sub][i]);
      }
    tmax = max8(tmax);
    float alpha = 1.0f;
    if (tmax > m_ref + kLazy) {                 // same decision in the 8 lanes of a head
      const float m_upd = fmaxf(m_ref, tmax);   // finite: the round's first tile holds a token
      alpha = fast_exp2(m_ref - m_upd);
      m_ref = m_upd;
      l_part *= alpha;
    }
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      float p0 = fast_exp2(sc[sub][0] - m_ref), p1 = fast_exp2(sc[sub][1] - m_ref);
      float p2 = fast_exp2(sc[sub][2] - m_ref), p3 = fast_exp2(sc[sub][3] - m_ref);
      float pdef = 0.f;
      if (newl[sub] >= 0 && newl[sub] < kTile) {  // wave-uniform: this tile holds the deferred token
        const int li = newl[sub] - slot;
        if (li == 0) { pdef = p0; p0 = 0.f; }
        if (li == 1) { pdef = p1; p1 = 0.f; }
        if (li == 2) { pdef = p2; p2 = 0.f; }
        if (li == 3) { pdef = p3; p3 = 0.f; }
        if (li >= 0 && li < 4 && o_hh < H) {
          pnew[(size_t)b * H + o_hh] = pdef;
          if (o_hh == 0) pnew_split[b] = s;
        }
      }
      u32x2_t hi, lo = {0, 0};
      hi[0] = cvt_pack(p0, p1, Tag{});
      hi[1] = cvt_pack(p2, p3, Tag{});
      float k0 = lo_to_f32(hi[0], Tag{}), k1 = hi_to_f32(hi[0], Tag{});
      float k2 = lo_to_f32(hi[1], Tag{}), k3 = hi_to_f32(hi[1], Tag{});
      if (SPLIT) {
        lo[0] = cvt_pack(p0 - k0, p1 - k1, Tag{});
        lo[1] = cvt_pack(p2 - k2, p3 - k3, Tag{});
        k0 += lo_to_f32(lo[0], Tag{});
        k1 += hi_to_f32(lo[0], Tag{});
        k2 += lo_to_f32(lo[1], Tag{});
        k3 += hi_to_f32(lo[1], Tag{});
      }
      l_part += (k0 + k1) + (k2 + k3) + pdef;   // the sum uses the values the MFMA will see
      u32x2_t* ph = (u32x2_t*)(Pbuf + ((sub * MT + o_mt) * 2 + 0) * 64 + o_lane) + o_tt;
      *ph = hi;
      if (SPLIT) *(ph + 2 * 64) = lo;
      if ((lane & 7) == 0) abuf[sub * 16 * MT + o_hh] = sub == 0 ? alpha : 1.0f;
    }
  }

  // (reference exponent, sum) of the heads this wave finalised.
  __device__ __forceinline__ void store_ml(float* part_ml) {
    const float l_tot = sum8(l_part);
    if (owner && (lane & 7) == 0 && o_hh < H) {
      const size_t pb = ((size_t)b * nsplit + s) * H + o_hh;
      part_ml[pb * 2 + 0] = m_ref;
      part_ml[pb * 2 + 1] = l_tot;
    }
  }
};

// Phase timers and per-tile time stamps for kernel studies (build with -DAP_KERNEL_TIMERS=2, or =1
// for the stamps alone, and set AP_DEBUG_ATTN: 4 = phase sums of workgroup (0,0) into the head of part_U, 8 = per-tile
// stamps into the bytes after the workspace, which the caller must have allocated).
#ifdef AP_KERNEL_TIMERS
#define AP_T_ENTRY                                                    \
  const unsigned long long t_entry_ = __builtin_readcyclecounter();   \
  const unsigned long long t_entry_rt_ = __builtin_amdgcn_s_memrealtime();
#define AP_T_START                                         \
  unsigned long long tm[8] = {0, 0, 0, 0, 0, 0, 0, 0};     \
  unsigned long long t0_ = __builtin_readcyclecounter();   \
  tm[0] = t0_ - t_entry_;                                  \
  if ((cx.dbg & 8) && cx.lane == 0) {                      \
    unsigned long long* o_ = uni_ptr(p.dbg_out) + 1024 + ((cx.b * cx.nsplit + cx.s) * 8 + cx.w) * 64; \
    o_[60] = t_entry_rt_;                                  \
    o_[61] = __builtin_amdgcn_s_memrealtime();             \
  }
#if AP_KERNEL_TIMERS >= 2
#define AP_TICK(k) { const unsigned long long now_ = __builtin_readcyclecounter(); tm[k] += now_ - t0_; t0_ = now_; }
#else
#define AP_TICK(k)
#endif
// in-loop stamps only from the first score wave (a sum wave counts its outstanding loads by hand,
// and a store in between would make it wait longer)
#define AP_T_STAMP(t)                                                                                    \
  if ((cx.dbg & 8) && cx.lane == 0 && (t) < 64 && (cx.w == 0 || (t) >= 60))                              \
    uni_ptr(p.dbg_out)[1024 + ((cx.b * cx.nsplit + cx.s) * 8 + cx.w) * 64 + (t)] = __builtin_amdgcn_s_memrealtime();
#define AP_T_REPORT                                                        \
  AP_T_STAMP(63)                                                           \
  if ((cx.dbg & 4) && cx.b == 0 && cx.s == 0 && cx.lane == 0) {            \
    unsigned long long* out_ = uni_ptr(p.dbg_out);                         \
    for (int k = 0; k < 8; ++k) out_[cx.w * 8 + k] = tm[k];                \
  }
#else
#define AP_T_ENTRY
#define AP_T_START
#define AP_TICK(k)
#define AP_T_STAMP(t)
#define AP_T_REPORT
#endif

template <class Tag, int MT, int RMAX, bool SPLIT, bool RAGGED, int Q>
__device__ __forceinline__ void score_role(const AttnParams& p) {
  constexpr bool I8 = Q != 0, I4 = Q == 2;
  constexpr uint32_t UB = I4 ? 32 : 64;                   // bytes of a row per unit (a scale block, or a k-step)
  constexpr uint32_t LB = I4 ? 8 : 16;                    // bytes of it per lane
  // a score wave owns "units" w, w+4, ... of the rank axis, 64 bytes of a row each:
  // 32-column k-steps for 16-bit storage, 64-column scale blocks (two k-steps) for int8
  constexpr bool TS = !RAGGED && !I8 && RMAX == 128;      // token-split mode (see WaveCtx)
  constexpr int NBW = (RMAX / 64 + 3) / 4;                // int8: scale blocks per score wave
  constexpr int NKW = TS ? RMAX / 32 : (I8 ? 2 * NBW : (RMAX / 32 + 3) / 4);   // score k-steps per score wave
  constexpr int NA = I8 ? NBW : NKW;                      // 16-byte row loads per 16-row half
  constexpr int Hp = MT * 16;
  AP_T_ENTRY
  WaveCtx<Tag, MT, SPLIT, RAGGED, Q, TS> cx;
  cx.init(p);
  float* part_ml = uni_ptr(p.part_ml);
  const int w = cx.w, n = cx.n, g = cx.g, r = cx.r, T = cx.T;
  const int nks = I8 ? r >> 6 : r >> 5;                   // all units
  // units of this wave: w, w+4, ... of every tile, or (token-split) all units of its tiles
  const int my_nks = TS ? nks : (nks > w ? (nks - w + 3) >> 2 : 0);
  const int ustep = TS ? 1 : 4, ufirst = TS ? 0 : w;      // unit index = ufirst + ustep * i
  // q' operands (B operand of the score MFMA): lane (h=n, g) holds columns 32ks+8g..+7
  // (int8: columns 64m+16g..+7 for a block's first k-step, 64m+16g+8..+15 for its second)
  const uint16_t* Qp = uni_ptr(p.Qp);
  u32x4_t qhi[NKW][MT];
  u32x4_t qlo[SPLIT ? NKW : 1][MT];
#pragma unroll
  for (int i = 0; i < NKW; ++i)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      u32x4_t z = {0, 0, 0, 0};
      qhi[i][mt] = z;
      if (SPLIT) qlo[i][mt] = z;
      const int unit = I8 ? i >> 1 : i;
#ifdef AP_KERNEL_TIMERS
      if (unit < my_nks && !(cx.dbg & 32)) {
#else
      if (unit < my_nks) {
#endif
        const int col = I8 ? (w + 4 * unit) * 64 + g * 16 + (i & 1) * 8 : (ufirst + ustep * i) * 32 + g * 8;
        const uint16_t* qrow = Qp + (((size_t)cx.b * 2) * Hp + (mt * 16 + n)) * r + col;
        qhi[i][mt] = *(const u32x4_t*)qrow;
        if (SPLIT) qlo[i][mt] = *(const u32x4_t*)(qrow + (size_t)Hp * r);
        if (I4) {                                          // the column order of code_row8_i4: 0,4,1,5,2,6,3,7
          const u32x4_t t = qhi[i][mt];
          qhi[i][mt][0] = __builtin_amdgcn_perm(t[2], t[0], 0x05040100u);
          qhi[i][mt][1] = __builtin_amdgcn_perm(t[2], t[0], 0x07060302u);
          qhi[i][mt][2] = __builtin_amdgcn_perm(t[3], t[1], 0x05040100u);
          qhi[i][mt][3] = __builtin_amdgcn_perm(t[3], t[1], 0x07060302u);
        }
      }
    }
  // C_k operands (A operand): lane (n, g) holds 16 bytes of token rows n, 16+n of the tile
  // per unit.  Per-sequence byte offsets fit 32 bits (checked on the host).
  const char* Ck_b = (const char*)uni_ptr(p.Ck) + (size_t)cx.b * uni(p.T_cap) * cx.row_bytes;
  // units this wave does not own re-read its first chunk (finite data times zero q'):
  // the loads carry no branches, so they issue back to back without waits between them
  const uint32_t lane_off = (uint32_t)(my_nks > 0 ? ufirst : 0) * UB + (uint32_t)g * LB;
  u32x4_t A[NA][2];
#pragma unroll
  for (int i = 0; i < NA; ++i) { u32x4_t z = {0, 0, 0, 0}; A[i][0] = z; A[i][1] = z; }
  uint32_t koff[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) koff[i] = i < my_nks ? (uint32_t)(i * ustep) * UB : 0u;
  auto load_piece = [](const char* src) -> u32x4_t {       // this lane's bytes of one unit of one row
    if constexpr (I4) {
      const u32x2_t h = *(const u32x2_t*)src;
      const u32x4_t v = {h[0], h[1], 0u, 0u};
      return v;
    } else {
      return *(const u32x4_t*)src;
    }
  };
  // int8: the key scale of the lane's row for every owned block (both halves of a packed
  // pair), and this wave's share of the tile's value scales, which the score waves pass to
  // the sum waves through LDS as [scale block][32 tokens]
  const int nsb = r >> 6;
  const uint16_t* Sk_b = I8 ? uni_ptr(p.Sk) + (size_t)cx.b * uni(p.T_cap) * nsb : nullptr;
  const uint16_t* Sv_b = I8 ? uni_ptr(p.Sv) + (size_t)cx.b * uni(p.T_cap) * nsb : nullptr;
  uint32_t ksc[I8 ? NBW : 1][2];
  uint16_t vsr[2] = {0, 0};
  const int vs_e0 = w * 64 + cx.lane;                      // entries vs_e0, vs_e0 + 256 of [block][token]
  auto load_scales = [&](int tile) {
    if constexpr (I8) {
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        int row;
        if (RAGGED) {
          row = cx.idxb[tile * kTile + 16 * tt + n];
        } else {
          row = cx.tok0(tile) + 16 * tt + n;
          row = row < T ? row : T - 1;
        }
        const uint16_t* sp_ = Sk_b + (size_t)row * nsb + (my_nks > 0 ? w : 0);
#pragma unroll
        for (int i = 0; i < NBW; ++i) {
          ksc[i][tt] = sp_[i < my_nks ? 4 * i : 0];
        }
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int e = vs_e0 + 256 * j;
        if (e < nsb * kTile) {
          int row;
          if (RAGGED) {
            row = cx.idxb[tile * kTile + (e & 31)];
          } else {
            row = cx.tok0(tile) + (e & 31);
            row = row < T ? row : T - 1;
          }
          vsr[j] = Sv_b[(size_t)row * nsb + (e >> 5)];
        }
      }
    }
  };
  auto load_A = [&](int tile, u32x4_t (&A)[NA][2]) {      // tile: local index in this split
    if (cx.dbg & 1) return;
    if (!RAGGED) {
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        int row = cx.tok0(tile) + 16 * tt + n;
        row = row < T ? row : T - 1;                      // rows beyond T are masked later
        const char* rp = Ck_b + ((uint32_t)row * cx.row_bytes + lane_off);
#pragma unroll
        for (int i = 0; i < NA; ++i) A[i][tt] = load_piece(rp + koff[i]);
      }
      load_scales(tile);
    } else {
      // gathered rows; only this wave's units below the tile's key rank are fetched (a
      // wave-uniform count, so a low-rank tile costs fewer requests, not just fewer distinct
      // bytes); the registers of the other units keep old values and are zeroed before the
      // product, like the columns beyond a rank that ends inside a 32-column k-step
      const int nks_t = I8 ? uni(cx.meta[4 * tile + 1]) >> 6 : (uni(cx.meta[4 * tile + 1]) + 31) >> 5;   // units of 64 bytes
      const int nlive_t = nks_t > w ? (nks_t - w + 3) >> 2 : 0;
      const uint32_t loff = (uint32_t)w * UB + (uint32_t)g * LB;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const int row = cx.idxb[tile * kTile + 16 * tt + n];
        const char* rp = Ck_b + ((uint32_t)row * cx.row_bytes + loff);
#pragma unroll
        for (int i = 0; i < NA; ++i)
          if (i < nlive_t) A[i][tt] = load_piece(rp + (uint32_t)i * 4u * UB);
      }
      load_scales(tile);
    }
  };
  if constexpr (TS) {
    // ---- token-split: this wave scores tiles w, w + 4, ... completely; four tiles per round
    const int rounds = (cx.ntl + 3) >> 2;
    if (w < cx.ntl) load_A(w, A);
    AP_T_START
    for (int it = 0; it < rounds; ++it) {
      const int lt = 4 * it + w;
      f32x4_t sp[MT][2];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) { f32x4_t z = {0.f, 0.f, 0.f, 0.f}; sp[mt][0] = z; sp[mt][1] = z; }
      score_tile<Tag, MT, SPLIT, NKW>(A, qhi, qlo, sp);     // a slot without a tile: masked below
      AP_TICK(1)
      if (lt + 4 < cx.ntl) load_A(lt + 4, A);               // lands while the round is finished
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        cx.xchg[(w * 16 * MT + mt * 16 + n) * 9 + g] = sp[mt][0];
        cx.xchg[(w * 16 * MT + mt * 16 + n) * 9 + 4 + g] = sp[mt][1];
      }
      wg_barrier();                                         // scores of the round's tiles ready
      AP_TICK(2)
      cx.finalize_softmax4(4 * it);
      AP_TICK(3)
      wg_barrier();                                         // weights of the round's tiles ready
      AP_TICK(4)
    }
    cx.store_ml(part_ml);
    AP_TICK(6)
    AP_T_REPORT
    return;
  }
  AP_T_START
  // One tile: scores from the rows in A, then the same registers take the rows of tile t + lead.
  auto tile_step = [&](int t, u32x4_t (&A)[NA][2], int lead) {
    AP_T_STAMP(t)
    f32x4_t sp[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) { f32x4_t z = {0.f, 0.f, 0.f, 0.f}; sp[mt][0] = z; sp[mt][1] = z; }
    if (RAGGED) {                                         // columns beyond the key rank count as zero
      const int rk_t = uni(cx.meta[4 * t + 1]);
#pragma unroll
      for (int i = 0; i < NA; ++i) {
        // 16-bit: this lane's eight columns of k-step w + 4i start at 32 (w + 4i) + 8 g, and ranks
        // are multiples of 8 there; int8: whole 64-column scale blocks
        const bool beyond = I8 ? (w + 4 * i) * 64 >= rk_t : (w + 4 * i) * 32 + g * 8 >= rk_t;
        if (beyond) {                                     // code 0 is the byte 0 for int8, the nibble 8 for 4-bit
          const uint32_t zc = I4 ? 0x88888888u : 0u;
          const u32x4_t z = {zc, zc, zc, zc};
          A[i][0] = z;
          A[i][1] = z;
        }
      }
    }
    if constexpr (I8) {
      // hand tile t's value scales to the sum waves (buffer t&1: its previous reader, the
      // weighted sum of tile t-2, ended before the barrier this wave passed in tile t-1)
      uint16_t* vs = cx.vsb + (t & 1) * nsb * kTile;
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (vs_e0 + 256 * j < nsb * kTile) vs[vs_e0 + 256 * j] = vsr[j];
      if (!(cx.dbg & 2)) score_tile_i8<MT, NBW, I4>(A, ksc, g, qhi, sp);
    } else {
      int nlive = NKW;
      if (RAGGED) {                                       // this wave's k-steps w, w + 4, ... below the key rank
        const int nks_t = (uni(cx.meta[4 * t + 1]) + 31) >> 5;
        nlive = nks_t > w ? (nks_t - w + 3) >> 2 : 0;
      }
      if (!(cx.dbg & 2)) score_tile<Tag, MT, SPLIT, NKW>(A, qhi, qlo, sp, nlive);
    }
    AP_TICK(1)
    if (t + lead < cx.ntl) load_A(t + lead, A);           // lands while the tile(s) in between are finished
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      cx.xchg[(w * 16 * MT + mt * 16 + n) * 9 + g] = sp[mt][0];
      cx.xchg[(w * 16 * MT + mt * 16 + n) * 9 + 4 + g] = sp[mt][1];
    }
    wg_barrier();                                         // partial scores of tile t ready
    AP_TICK(2)
    cx.finalize_softmax(cx.tile_valid(t), cx.tile_new(t), t);
    AP_TICK(3)
    wg_barrier();                                         // weights of tile t ready
    AP_TICK(4)
  };
  if (cx.ntl > 0) load_A(0, A);
  for (int t = 0; t < cx.ntl; ++t) tile_step(t, A, 1);
  AP_T_STAMP(62)
  cx.store_ml(part_ml);
  AP_TICK(6)
  AP_T_REPORT
}

template <class Tag, int MT, int RMAX, bool SPLIT, bool RAGGED, int Q>
__device__ __forceinline__ void sum_role(const AttnParams& p) {
  constexpr bool I8 = Q != 0, I4 = Q == 2;
  constexpr bool TS = !RAGGED && !I8 && RMAX == 128;              // token-split mode (see WaveCtx)
  constexpr int RB = I4 ? RMAX / 2 : (I8 ? RMAX : 2 * RMAX);      // bytes of a coefficient row at most
  // column groups of 256 bytes (16-bit, int8: 128 / 256 columns, the wave owns 64 bytes of each);
  // 4-bit: groups of four 64-column scale blocks (128 bytes), one block per wave
  constexpr int NGRP = I4 ? (RMAX / 64 + 3) / 4 : (RB + 255) / 256;
  constexpr int NJ = I8 ? 4 : 2;                                  // accumulator tiles per group
  constexpr int MAXBLK = (kHalf * (RB / 16 + 1) + 63) / 64;       // 1 KiB blocks per ring unit
  constexpr int NSLOT = (MAXBLK + 3) / 4;
  AP_T_ENTRY
  WaveCtx<Tag, MT, SPLIT, RAGGED, Q, TS> cx;
  cx.init(p);
  float* part_U = uni_ptr(p.part_U);
  float* part_ml = uni_ptr(p.part_ml);
  const int n = cx.n, g = cx.g, r = cx.r, lane = cx.lane;
  const int cp = cx.w - 4;                                // which 64 bytes of every group
  const int RT = cx.nh >> 1;                              // ring capacity in tiles

  // ---- this wave's share of a C_v ring unit: 1 KiB blocks cp, cp+4, ...; per lane the
  //      row and the byte offset of its 16-byte chunk from the unit's first row
  const int cpr = (int)cx.row_bytes >> 4;
  const int tot_chunks = kHalf * (cpr + 1);
  uint32_t slot_off[NSLOT];
  uint32_t slot_row[(NSLOT + 3) / 4];
#pragma unroll
  for (int k = 0; k < (NSLOT + 3) / 4; ++k) slot_row[k] = 0;
  int n_issue = 0;
#pragma unroll
  for (int k = 0; k < NSLOT; ++k) {
    const int blk = cp + 4 * k;
    slot_off[k] = 0;
    if (blk < cx.nblk) {
      ++n_issue;
      const int L = blk * 64 + lane;
      int row = L / (cpr + 1);
      int c = L - row * (cpr + 1);
      if (L >= tot_chunks) { row = 0; c = 0; }   // tail of the last block: harmless duplicate
      if (c == cpr) c = 0;                        // pad chunk: harmless duplicate
      slot_off[k] = (uint32_t)row * cx.row_bytes + (uint32_t)(c * 16);
      slot_row[k >> 2] |= (uint32_t)row << (8 * (k & 3));
    }
  }
  const char* Cv_b = (const char*)uni_ptr(p.Cv) + (size_t)cx.b * uni(p.T_cap) * cx.row_bytes;
  // RAGGED: a gathered tile sits in its ring slots packed to its own value rank: 16 rows of
  // (chunks below the rank + one pad chunk), so a low-rank tile takes fewer 1 KiB requests and
  // not just fewer distinct bytes.  16-byte chunks of a row below the rank of local tile lt:
  auto tile_chunks = [&](int lt) -> int {
    const int rv = uni(cx.meta[4 * lt + 2]);
    int c = I4 ? (rv + 31) >> 5 : (I8 ? (rv + 15) >> 4 : (rv + 7) >> 3);
    c = c < 1 ? 1 : c;
    return c < cpr ? c : cpr;
  };
  // ... and this wave's requests per 16-row unit of such a tile (blocks cp, cp + 4, ...)
  auto tile_requests = [&](int lt) -> int {
    const int nb = (kHalf * (tile_chunks(lt) + 1) + 63) >> 6;
    return nb > cp ? (nb - cp + 3) >> 2 : 0;
  };
  // both 16-row units of local tile lt into ring slots 2*(lt % RT), +1
  auto issue_tile = [&](int lt) {
    if (cx.dbg & 1) return;
    const int slot0 = 2 * (lt % RT);
    if (RAGGED) {
      const int cprt = tile_chunks(lt), cw = cprt + 1, tot = kHalf * cw;
      const int nb = (tot + 63) >> 6;
      // chunk L of a unit is (row L / cw, chunk L % cw): L < 1344 and cw <= 81, so the quotient
      // is exact as (L * ceil(2^20 / cw)) >> 20
      const uint32_t magic = ((1u << 20) + (uint32_t)cw - 1u) / (uint32_t)cw;
#pragma nounroll
      for (int half = 0; half < 2; ++half) {
        char* dst = cx.ring + (slot0 + half) * cx.unit_bytes;
        const int* ix = cx.idxb + lt * kTile + half * kHalf;
#pragma unroll
        for (int k = 0; k < NSLOT; ++k) {
          const int blk = cp + 4 * k;
          if (blk < nb) {                                     // wave-uniform
            const uint32_t L = (uint32_t)(blk * 64 + lane);
            uint32_t row = (L * magic) >> 20;
            uint32_t c = L - row * (uint32_t)cw;
            if (L >= (uint32_t)tot) { row = 0; c = 0; }       // tail of the last block: harmless duplicate
            if (c == (uint32_t)cprt) c = 0;                   // pad chunk: harmless duplicate
            int tokv = ix[row];
            tokv = tokv < cx.Tv ? tokv : cx.Tv - 1;           // a deferred row is not there yet: weight 0
            dma16(Cv_b + ((uint32_t)tokv * cx.row_bytes + c * 16u), dst + blk * 1024);
          }
        }
      }
      return;
    }
#pragma nounroll
    for (int half = 0; half < 2; ++half) {
      const int tok_u = cx.tok0(lt) + half * kHalf;
      char* dst = cx.ring + (slot0 + half) * cx.unit_bytes;
      const uint32_t base = (uint32_t)tok_u * cx.row_bytes;
      const int vlim = cx.Tv;
      if (tok_u + kHalf <= vlim) {
#pragma unroll
        for (int k = 0; k < NSLOT; ++k) {
          const int blk = cp + 4 * k;
          if (blk < cx.nblk) dma16(Cv_b + (base + slot_off[k]), dst + blk * 1024);
        }
      } else {                                     // rows that do not exist: repeat the last that does
#pragma unroll
        for (int k = 0; k < NSLOT; ++k) {
          const int blk = cp + 4 * k;
          if (blk < cx.nblk) {
            const int row = (int)((slot_row[k >> 2] >> (8 * (k & 3))) & 0xffu);
            uint32_t off = base + slot_off[k];
            if (tok_u + row >= vlim) off -= (uint32_t)(tok_u + row - (vlim - 1)) * cx.row_bytes;
            dma16(Cv_b + off, dst + blk * 1024);
          }
        }
      }
    }
  };
  // Only the first tile is requested up front: the rest of the ring is filled once the score
  // waves have their first tile, so the folded query and the first key tile (which everything
  // waits for) are not queued behind value rows that are needed later.
  if (cx.ntl > 0) issue_tile(0);

  f32x4_t U[NGRP][NJ][MT];
#pragma unroll
  for (int i = 0; i < NGRP; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) { f32x4_t z = {0.f, 0.f, 0.f, 0.f}; U[i][j][mt] = z; }
  AP_T_START
  if constexpr (TS) {
    // ---- token-split: four tiles per round (the host sizes the ring for at least eight)
    const int rounds = (cx.ntl + 3) >> 2;
    for (int it = 0; it < rounds; ++it) {
      wg_barrier();          // scores of this round ready; every sum wave is past the last round
      AP_TICK(2)
      // tiles requested so far: 0 (before the loop), then up to 4 it + RT - 1
      if (it == 0) {
#pragma nounroll
        for (int lt = 1; lt < RT && lt < cx.ntl; ++lt) issue_tile(lt);
      } else {
#pragma nounroll
        for (int lt = 4 * it + RT - 4; lt < 4 * it + RT && lt < cx.ntl; ++lt) issue_tile(lt);   // refill the last round's slots
      }
      cx.finalize_softmax4(4 * it);
      AP_TICK(3)
      {
        // this round's tiles must have landed; those requested beyond it may stay in flight
        int upto = 4 * it + RT;
        upto = upto < cx.ntl ? upto : cx.ntl;
        int need = 4 * it + 4;
        need = need < cx.ntl ? need : cx.ntl;
        wait_vmcnt((upto - need) * 2 * n_issue);
      }
      wg_barrier();          // weights of this round ready; its rows visible to every wave
      AP_TICK(4)
#pragma unroll
      for (int sub = 0; sub < 4; ++sub) {
        const int t = 4 * it + sub;
        if (t < cx.ntl) {
          u32x4_t Phi[MT], Plo[MT];
          float alpha[MT];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            alpha[mt] = cx.abuf[sub * 16 * MT + mt * 16 + n];
            Phi[mt] = cx.Pbuf[((sub * MT + mt) * 2 + 0) * 64 + lane];
            if (SPLIT) Plo[mt] = cx.Pbuf[((sub * MT + mt) * 2 + 1) * 64 + lane];
            else { u32x4_t z = {0, 0, 0, 0}; Plo[mt] = z; }
          }
          const int slot0 = 2 * (t % RT);
          const char* vA = cx.ring + slot0 * cx.unit_bytes + (4 * g) * cx.pitch + cp * 64 + n * 4;
          const char* vB = vA + cx.unit_bytes;
          wsum_tile<Tag, MT, SPLIT, NGRP>(vA, vB, cx.pitch, r - cp * 32, n, Phi, Plo, alpha, U);
        }
      }
      AP_TICK(5)
    }
  } else {
  for (int t = 0; t < cx.ntl; ++t) {
    AP_T_STAMP(t)
    wg_barrier();            // partial scores of tile t ready; every sum wave is past tile t-1
    AP_TICK(2)
    if (t == 0) {
#pragma nounroll
      for (int lt = 1; lt < RT && lt < cx.ntl; ++lt) issue_tile(lt);
    } else if (t - 1 + RT < cx.ntl) {
      issue_tile(t - 1 + RT);                                    // refill tile t-1's slots
    }
    cx.finalize_softmax(cx.tile_valid(t), cx.tile_new(t), t);
    AP_TICK(3)
    {
      // tile t's rows must have landed; the tiles issued after it may stay in flight
      int later = cx.ntl - t - 1;
      later = later < RT - 1 ? later : RT - 1;
      if (RAGGED) {
        int pending = 0;
        for (int lt = t + 1; lt <= t + later; ++lt) pending += 2 * tile_requests(lt);
        wait_vmcnt(pending);
      } else {
        wait_vmcnt(later * 2 * n_issue);
      }
    }
    wg_barrier();            // weights of tile t ready; tile t's rows visible to every wave
    AP_TICK(4)
    u32x4_t Phi[MT], Plo[MT];
    float alpha[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      alpha[mt] = cx.abuf[mt * 16 + n];
      Phi[mt] = cx.Pbuf[(mt * 2 + 0) * 64 + lane];
      if (SPLIT) Plo[mt] = cx.Pbuf[(mt * 2 + 1) * 64 + lane];
      else { u32x4_t z = {0, 0, 0, 0}; Plo[mt] = z; }
    }
    // lane (n, g): token rows 4g..4g+3 (and 16+4g..), dword n of this wave's 64 bytes
    const int slot0 = 2 * (t % RT);
    const int pitch_t = RAGGED ? (tile_chunks(t) + 1) * 16 : cx.pitch;
    const char* vA = cx.ring + slot0 * cx.unit_bytes + (4 * g) * pitch_t + cp * 64 + n * 4;
    const char* vB = vA + cx.unit_bytes;
    if constexpr (I8) {
      f32x4_t P32[MT][2];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        P32[mt][0] = __builtin_bit_cast(f32x4_t, Phi[mt]);
        P32[mt][1] = __builtin_bit_cast(f32x4_t, cx.Pbuf[(mt * 2 + 1) * 64 + lane]);
      }
      if constexpr (I4) {
        // the 4-bit reader places its own block and dword: take the wave's and the lane's offsets off
        if (!(cx.dbg & 2))
          wsum_tile_i4<MT, NGRP>(vA - cp * 64 - n * 4, vB - cp * 64 - n * 4, pitch_t, RAGGED ? uni(cx.meta[4 * t + 2]) : r, cp, n, g,
                                 cx.vsb + (t & 1) * (r >> 6) * kTile, P32, alpha, U);
      } else {
        if (!(cx.dbg & 2))
          wsum_tile_i8<MT, NGRP>(vA, vB, pitch_t, RAGGED ? uni(cx.meta[4 * t + 2]) : r, cp, g,
                                 cx.vsb + (t & 1) * (r >> 6) * kTile, P32, alpha, U);
      }
    } else {
      if (!(cx.dbg & 2))
        wsum_tile<Tag, MT, SPLIT, NGRP>(vA, vB, pitch_t,
                                        (RAGGED ? uni(cx.meta[4 * t + 2]) : r) - cp * 32, n, Phi, Plo,
                                        alpha, U);
    }
    AP_TICK(5)
  }
  }
  AP_T_STAMP(62)
  // U of this split, straight from the accumulators.  U[i][j][mt][e] is element (head 16mt+n,
  // column 128i + 32cp + 8g + 2e + j) (int8: column 256i + 64cp + 16g + 4e + j): a lane owns
  // NJ*4 consecutive columns of one head per column group, stored as 16-byte pieces; the four
  // lanes g = 0..3 of a head together cover a full 128-byte (int8: 256-byte) run.
#ifdef AP_KERNEL_TIMERS
  if (!(cx.dbg & 16))
#endif
  {
    float* ubase = part_U + ((size_t)cx.b * cx.nsplit + cx.s) * cx.H * r;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int head = mt * 16 + n;
      if (head < cx.H) {
        float* urow = ubase + (size_t)head * r;
#pragma unroll
        for (int i = 0; i < NGRP; ++i) {
          const int col0 = I8 ? i * 256 + cp * 64 + g * 16 : i * 128 + cp * 32 + g * 8;
          if constexpr (I4) {
            // accumulator row 4g + e of tile j of block 4 i + cp is column 64 (4 i + cp) + 32 (g & 1)
            // + 8 e + 4 (g >> 1) + j: the four j of one e are consecutive
            const int cb = (4 * i + cp) * 64 + (g & 1) * 32 + (g >> 1) * 4;
            if (cb < r) {
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const f32x4_t v = {U[i][0][mt][e], U[i][1][mt][e], U[i][2][mt][e], U[i][3][mt][e]};
                *(f32x4_t*)(urow + cb + 8 * e) = v;
              }
            }
          } else if (col0 < r) {
            if constexpr (I8) {
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const f32x4_t v = {U[i][0][mt][e], U[i][1][mt][e], U[i][2][mt][e], U[i][3][mt][e]};
                *(f32x4_t*)(urow + col0 + 4 * e) = v;
              }
            } else {
#pragma unroll
              for (int e2 = 0; e2 < 2; ++e2) {
                const f32x4_t v = {U[i][0][mt][2 * e2], U[i][1][mt][2 * e2], U[i][0][mt][2 * e2 + 1],
                                   U[i][1][mt][2 * e2 + 1]};
                *(f32x4_t*)(urow + col0 + 4 * e2) = v;
              }
            }
          }
        }
      }
    }
  }
  cx.store_ml(part_ml);
  AP_TICK(6)
  AP_T_REPORT
}
#undef AP_TICK
#undef AP_T_ENTRY
#undef AP_T_START
#undef AP_T_STAMP
#undef AP_T_REPORT

template <class Tag, int MT, int RMAX, bool SPLIT, bool RAGGED, int Q>
__device__ __noinline__ void score_role_call(const AttnParams& p) {
  score_role<Tag, MT, RMAX, SPLIT, RAGGED, Q>(p);
}
template <class Tag, int MT, int RMAX, bool SPLIT, bool RAGGED, int Q>
__device__ __noinline__ void sum_role_call(const AttnParams& p) {
  sum_role<Tag, MT, RMAX, SPLIT, RAGGED, Q>(p);
}

template <class Tag, int MT, int RMAX, bool SPLIT, bool RAGGED, int Q>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
attn_partial(const AttnParams p) {
  {
    int b, s;
    wg_coords(p.nsplit, p.xcd_aware, b, s);
    if (b >= p.B) return;
  }
  // The roles are inlined: called as functions they would spill their callee-saved registers
  // and read the launch parameters back from a scratch copy, a dozen serial memory round trips
  // at the start of every wave.  Only the largest shape (64 heads at rank 640), whose two roles
  // do not fit one register allocation without spilling inside the tile loop, keeps the calls.
  constexpr bool kOutline = MT == 4 && RMAX > 512;
  if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) < 4) {
    if constexpr (kOutline) score_role_call<Tag, MT, RMAX, SPLIT, RAGGED, Q>(p);
    else score_role<Tag, MT, RMAX, SPLIT, RAGGED, Q>(p);
  } else {
    if constexpr (kOutline) sum_role_call<Tag, MT, RMAX, SPLIT, RAGGED, Q>(p);
    else sum_role<Tag, MT, RMAX, SPLIT, RAGGED, Q>(p);
  }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
// Splits of the token axis: enough workgroups to cover every CU once, never finer
// than one 32-token tile.  The count does not depend on the device, so the workspace
// query needs no GPU.
constexpr int kMaxTilesPerSplit = 128;   // bounds the LDS index table of rank-ragged launches
constexpr int kMaxGroups = 8;
constexpr int kInlineMergeSplits = 16;   // more splits than this are merged by their own kernel
constexpr int kFusedInlineSplits = 16;   // the same limit inside a fused step (measured: merging
                                         // 16 splits inline saves 6-8 us, merging 32 costs 5)

int choose_nsplit(int B, int T) {
  const int ntiles = (T + kTile - 1) / kTile;
  int s = 256 / B;                         // one workgroup per CU at most: a second, partial round
                                           // of workgroups would double the kernel's time
  const int by_table = (ntiles + kMaxGroups + kMaxTilesPerSplit - 1) / kMaxTilesPerSplit;
  if (s < by_table) {
    // more workgroups than CUs: whole rounds of 256 (a partial last round would run alone)
    s = by_table;
    int g = 256, x = B;
    while (x) { const int t = g % x; g = x; x = t; }          // gcd(256, B)
    const int step = 256 / g;
    const int s_up = (s + step - 1) / step * step;
    if (s_up <= 2 * s) s = s_up;
  }
  if (s > ntiles) s = ntiles;
  if (s < 1) s = 1;
  return s;
}

struct WsLayout {
  size_t qp, ml, u, po, pn, mml, mu, total;
};
WsLayout ws_layout(int B, int H, int d, int T, int r) {
  const int Hp = (H + 15) / 16 * 16;
  const int S = choose_nsplit(B, T);
  WsLayout w;
  w.qp = 0;
  size_t off = round_up((size_t)B * 2 * Hp * r * 2, 256);
  w.ml = off;
  off += round_up((size_t)B * S * H * 2 * 4, 256);
  w.u = off;
  off += round_up((size_t)B * S * H * r * 4, 256);
  w.po = off;                              // per-row-block output sums of a fused step
  off += round_up((size_t)B * expand_row_blocks(B, r) * H * d * 4, 256);
  w.pn = off;                              // the newest token's softmax weights of a fused step
  off += round_up((size_t)B * H * 4 + (size_t)B * 4, 256);   // ... and the split that holds it
  w.mml = off;                             // many splits: merged (m, l) and U as a single split
  off += round_up((size_t)B * H * 2 * 4, 256);
  w.mu = off;
  off += S > kInlineMergeSplits ? round_up((size_t)B * H * r * 4, 256) : 0;
  w.total = off;
  return w;
}

template <class Tag, int MT, int RMAX, bool SPLIT, bool RAGGED, int Q>
ap_status launch_attn(AttnParams p, int B, hipStream_t stream) {
  constexpr bool I8 = Q != 0;
  const int cpr = (Q == 2 ? p.r / 2 : (I8 ? p.r : 2 * p.r)) / 16;
  const size_t unit = (size_t)((kHalf * (cpr + 1) + 63) / 64) * 1024;
  constexpr bool TS = !RAGGED && !I8 && RMAX == 128;
  constexpr int NSUB = TS ? 4 : 1;
  size_t fixed = (size_t)4 * 16 * MT * 9 * 16 + (size_t)NSUB * MT * 2 * 64 * 16 + (size_t)NSUB * MT * 16 * 4;
  if (I8) fixed += (size_t)2 * (p.r / 64) * kTile * 2;     // value scales of two tiles
  if (RAGGED) {
    // every group may end in a partial tile; tiles are dealt round-robin to the splits
    const int ntiles_max = (p.T + kTile - 1) / kTile + p.F;
    p.ntl_cap = (ntiles_max + p.nsplit - 1) / p.nsplit;
    fixed += (size_t)p.ntl_cap * (kTile + 4) * 4;
  }
  const size_t budget = 160 * 1024;
  AP_REQUIRE(fixed + 2 * unit <= budget, AP_ERR_UNSUPPORTED,
             "ap_decode_attn: H=%d r=%d needs more LDS than 160 KiB", p.H, p.r);
  int nh = (int)((budget - fixed) / unit);
  if (TS) {
    // four tiles are consumed per round: a ring of 8 or 12 tiles (16-row units come in pairs)
    nh = nh >= 24 ? 24 : 16;
    AP_REQUIRE(fixed + (size_t)nh * unit <= budget, AP_ERR_UNSUPPORTED,
               "ap_decode_attn: H=%d r=%d needs more LDS than 160 KiB", p.H, p.r);
  } else {
    if (nh > 12) nh = 12;
    nh &= ~1;
  }
  p.nh = nh;
  size_t lds = (size_t)nh * unit + fixed;
  auto kern = attn_partial<Tag, MT, RMAX, SPLIT, RAGGED, Q>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)budget);
    if (e != hipSuccess) {
      set_error("hipFuncSetAttribute: %s", hipGetErrorString(e));
      return AP_ERR_HIP;
    }
    attr_set = true;
  }
  p.B = B;
  p.xcd_aware = B % 8 == 0 ? 1 : 0;
  hipEvent_t ev0, ev1;
  if (prof_events(&ev0, &ev1))             // timing on: the events carry this launch's own start and end
    hipExtLaunchKernelGGL(kern, dim3(B * p.nsplit), dim3(512), (uint32_t)lds, stream, ev0, ev1, 0u, p);
  else
    hipLaunchKernelGGL(kern, dim3(B * p.nsplit), dim3(512), lds, stream, p);
  return AP_OK;
}

template <class Tag, bool SPLIT>
ap_status dispatch_attn(const AttnParams& p, int B, hipStream_t stream) {
  const int nw = (p.H + 15) / 16;
  if constexpr (!SPLIT) {                 // fp16 arithmetic: int8 coefficients ride on it
    if (p.Sk && p.qbits == 4) {
      switch (nw) {
#define AP_CASE4(NWV)                                                                  \
  case NWV:                                                                            \
    if (p.bucket_idx)                                                                  \
      return p.r <= 512 ? launch_attn<Tag, NWV, 512, false, true, 2>(p, B, stream)     \
                        : launch_attn<Tag, NWV, 640, false, true, 2>(p, B, stream);    \
    return p.r <= 512 ? launch_attn<Tag, NWV, 512, false, false, 2>(p, B, stream)      \
                      : launch_attn<Tag, NWV, 640, false, false, 2>(p, B, stream);
        AP_CASE4(1) AP_CASE4(2) AP_CASE4(3) AP_CASE4(4)
#undef AP_CASE4
      }
    }
    if (p.Sk) {
      switch (nw) {
#define AP_CASE8(NWV)                                                                     \
  case NWV:                                                                               \
    if (p.bucket_idx)                                                                     \
      return p.r <= 256   ? launch_attn<Tag, NWV, 256, false, true, true>(p, B, stream)   \
             : p.r <= 512 ? launch_attn<Tag, NWV, 512, false, true, true>(p, B, stream)   \
                          : launch_attn<Tag, NWV, 640, false, true, true>(p, B, stream);  \
    return p.r <= 256   ? launch_attn<Tag, NWV, 256, false, false, true>(p, B, stream)    \
           : p.r <= 512 ? launch_attn<Tag, NWV, 512, false, false, true>(p, B, stream)    \
                        : launch_attn<Tag, NWV, 640, false, false, true>(p, B, stream);
        AP_CASE8(1) AP_CASE8(2) AP_CASE8(3) AP_CASE8(4)
#undef AP_CASE8
      }
    }
  }
#define AP_CASE(NWV)                                                                  \
  case NWV:                                                                           \
    if (p.bucket_idx)                                                                 \
      return p.r <= 256   ? launch_attn<Tag, NWV, 256, SPLIT, true, false>(p, B, stream)     \
             : p.r <= 512 ? launch_attn<Tag, NWV, 512, SPLIT, true, false>(p, B, stream)     \
                          : launch_attn<Tag, NWV, 640, SPLIT, true, false>(p, B, stream);    \
    if (p.r <= 128) return launch_attn<Tag, NWV, 128, SPLIT, false, false>(p, B, stream);    \
    return p.r <= 256   ? launch_attn<Tag, NWV, 256, SPLIT, false, false>(p, B, stream)      \
           : p.r <= 512 ? launch_attn<Tag, NWV, 512, SPLIT, false, false>(p, B, stream)      \
                        : launch_attn<Tag, NWV, 640, SPLIT, false, false>(p, B, stream);
  switch (nw) {
    AP_CASE(1) AP_CASE(2) AP_CASE(3) AP_CASE(4)
  }
#undef AP_CASE
  set_error("ap_decode_attn: H=%d unsupported", p.H);
  return AP_ERR_UNSUPPORTED;
}

template <class Tag, bool SPLIT>
ap_status run_decode(const DecodeArgs& a) {
  const int Hp = (a.H + 15) / 16 * 16;
  // A fused step scores all T tokens in attn_partial but leaves the newest
  // token's value row to the expansion pass over B_v, which produces that row and adds its
  // contribution: B_v is read once per step instead of twice.
  const int Hkv = a.H_kv;
  const int HDkv = Hkv * a.d;              // hidden columns of the cache and of the basis rows
  // That pays when a pass over the value bases is long: the expansion then writes and re-reads
  // per-row-block sums and needs a launch more, which costs more than streaming a small B_v a
  // second time next to B_k (measured: 47 against 58 us at rank 64, 103 against 110 us at B=32,
  // r=320; 312 against 361 us at B=64, r=640).
  const int64_t v_bytes = (int64_t)(a.basis_batch_stride ? a.B : 1) * a.r * HDkv * 2;
  const int64_t v_min = fused_value_min_bytes();
  const bool v_long = v_min >= 0 ? v_bytes >= v_min
                                 : v_bytes >= (128ll << 20) || (a.r >= 512 && v_bytes >= (96ll << 20));
  const bool quant = a.dt_coef == AP_I8 || a.dt_coef == AP_I4;
  const bool ragged = a.rank_k || a.rank_v;
  // (with per-token ranks only on the two-role kernel, whose gathered tiles know the newest token)
  const bool one_pass_v = a.v_new && a.T >= 2 && Hkv == a.H && v_long &&
                          !(ragged && attn_small_applies(a.H, a.r, a.T, false));
  const bool small = !quant && attn_small_applies(a.H, a.r, a.T, one_pass_v);
  int* pnew_split = (int*)((char*)a.workspace + ws_layout(a.B, a.H, a.d, a.T, a.r).pn + (size_t)a.B * a.H * 4);
  const int S = choose_nsplit(a.B, a.T);     // the same count for both kernels (twice the splits for
                                             // the small-rank kernel measured slower)
  const WsLayout wl = ws_layout(a.B, a.H, a.d, a.T, a.r);
  char* ws = (char*)a.workspace;
  uint16_t* Qp = (uint16_t*)(ws + wl.qp);
  float* ml = (float*)(ws + wl.ml);
  float* U = (float*)(ws + wl.u);
  // fold (and, for a fused step, the append of the key row in the same pass over B_k)
  ap_status st;
  // a value row that the expansion pass does not produce is appended in the same launch as the
  // key row (second job of the basis pass)
  const bool pair_v = a.v_new && !one_pass_v && a.k_new;
  if (Hkv == a.H) {
    st = launch_basis_rows(a.dt, a.Bk, a.basis_batch_stride, a.k_new, a.q, (void*)a.Ck, Qp, a.B, a.H, Hp,
                           a.d, a.H * a.d, a.r, a.T - 1, a.T_cap, a.sm_scale * kLog2e, a.stream,
                           pair_v ? a.Bv : nullptr, pair_v ? a.v_new : nullptr, pair_v ? (void*)a.Cv : nullptr);
  } else {
    // grouped queries: the key row is appended by a pass of its own over the (small) basis,
    // the fold runs per query head
    st = AP_OK;
    if (a.k_new)
      st = launch_basis_rows(a.dt, a.Bk, a.basis_batch_stride, a.k_new, nullptr, (void*)a.Ck, nullptr,
                             a.B, 0, 0, 8, HDkv, a.r, a.T - 1, a.T_cap, 1.0f, a.stream,
                             pair_v ? a.Bv : nullptr, pair_v ? a.v_new : nullptr, pair_v ? (void*)a.Cv : nullptr);
    if (st != AP_OK) return st;
    st = launch_fold_heads(a.dt, a.Bk, a.basis_batch_stride, a.q, Qp, a.B, a.H, Hkv, Hp, a.d, a.r,
                           a.sm_scale * kLog2e, a.stream);
  }
  if (st != AP_OK) return st;
  if (a.v_new && !one_pass_v && !pair_v) {
    st = launch_basis_rows(a.dt, a.Bv, a.basis_batch_stride, a.v_new, nullptr, (void*)a.Cv, nullptr,
                           a.B, 0, 0, 8, HDkv, a.r, a.T - 1, a.T_cap, 1.0f, a.stream);
    if (st != AP_OK) return st;
  }
  AttnParams p{};
  p.Qp = Qp;
  p.Ck = (const uint16_t*)a.Ck;
  p.Cv = (const uint16_t*)a.Cv;
  p.part_ml = ml;
  p.part_U = U;
  p.T = a.T; p.T_cap = a.T_cap; p.r = a.r; p.H = a.H; p.nsplit = S;
  p.scores = a.scores;
  p.defer_v = one_pass_v ? 1 : 0;
  p.pnew = (float*)(ws + wl.pn);
  p.pnew_split = pnew_split;
  if (quant) {
    p.Sk = (const uint16_t*)a.scale_k;
    p.Sv = (const uint16_t*)a.scale_v;
    p.qbits = a.dt_coef == AP_I4 ? 4 : 8;
  }
  if (a.rank_k || a.rank_v) {             // rank-ragged: walk the group lists
    p.rank_k = a.rank_k;
    p.rank_v = a.rank_v;
    p.bucket_off = a.bucket_off;
    p.bucket_idx = a.bucket_idx;
    p.F = a.F;
  }
#ifdef AP_KERNEL_TIMERS
  if (const char* e = getenv("AP_DEBUG_ATTN")) p.dbg = atoi(e);
  p.dbg_out = (unsigned long long*)U;   // timers overwrite the head of part_U
  if (p.dbg & 8) p.dbg_out = (unsigned long long*)(ws + wl.total);   // caller allocated extra bytes
#endif
  // small uniform ranks take the kernel whose waves work alone on whole tiles (attn_small.hip);
  // everything else the two-role kernel
  if (small)
    st = launch_attn_small(a.dt, Qp, a.Ck, a.Cv, ml, U, (float*)(ws + wl.pn), a.scores, a.rank_k, a.rank_v,
                           a.bucket_off, a.bucket_idx, a.F, a.B, a.H, a.T, a.T_cap, a.r, S, one_pass_v, a.stream);
  else
    st = dispatch_attn<Tag, SPLIT>(p, a.B, a.stream);
  if (st != AP_OK) return st;
  int S_exp = S;
  // many splits (small batches): merge_expand takes at most kInlineMergeSplits, so they are merged
  // by a kernel of their own first; the fused step's expansion merges up to kFusedInlineSplits
  // itself (its row blocks partition the columns, so no column is merged twice)
  if (S > (one_pass_v ? kFusedInlineSplits : kInlineMergeSplits)) {
    float* ml1 = (float*)(ws + wl.mml);
    float* U1 = (float*)(ws + wl.mu);
    st = launch_merge_splits(ml, U, ml1, U1, one_pass_v ? (float*)(ws + wl.pn) : nullptr,
                             one_pass_v && !small ? pnew_split : nullptr, a.B, a.H, a.r, S, a.stream);
    if (st != AP_OK) return st;
    ml = ml1;
    U = U1;
    S_exp = 1;
  }
  if (one_pass_v)
    st = launch_expand_append(a.dt, a.dt_out == AP_F32, a.Bv, a.basis_batch_stride, a.v_new,
                              (void*)a.Cv, ml, U, (const float*)(ws + wl.pn),
                              !small && S_exp > 1 ? pnew_split : nullptr, a.rank_v, (float*)(ws + wl.po),
                              a.out, a.lse, a.B, a.H, a.d, a.r, a.T, a.T_cap, S_exp, a.stream);
  else
    st = launch_merge_expand(a.dt, a.dt_out == AP_F32, ml, U, a.Bv, a.basis_batch_stride, a.out, a.lse,
                             a.B, a.H, Hkv, a.d, a.r, S_exp, a.stream);
  if (st != AP_OK) return st;
  return check_launch("ap_decode_attn");
}

}  // namespace

size_t decode_mfma_workspace(int B, int H, int d, int T, int r, ap_dtype dt) {
  (void)dt;
  return ws_layout(B, H, d, T, r).total;
}

ap_status launch_decode_mfma(const DecodeArgs& a) {
  AP_REQUIRE(a.B <= 65535, AP_ERR_UNSUPPORTED, "ap_decode_attn: B must be <= 65535");
  AP_REQUIRE(basis_rows_applies(a.H_kv * a.d, a.B), AP_ERR_UNSUPPORTED,
             "ap_decode_attn: H*d must be a multiple of 8 and <= 8192");
  AP_REQUIRE((int64_t)a.T_cap * a.r * 2 < (1ll << 32), AP_ERR_UNSUPPORTED,
             "ap_decode_attn: one sequence's coefficients must stay below 4 GiB");
  return a.dt == AP_F16 ? run_decode<F16Tag, false>(a) : run_decode<BF16Tag, true>(a);
}

}  // namespace ap
