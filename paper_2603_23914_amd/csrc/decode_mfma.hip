// Decode attention over fp16 / bf16 coefficients on the matrix cores (gfx950).
//
// Paper Alg. 1 (partial decompression, scores, softmax, output) with the
// decompression matrices absorbed by associativity, so K and V are never rebuilt:
//   fold:    q'[h,j]  = sm_scale*log2(e) * sum_i Bk[j, h*d+i] q[h,i]      (kernel fold_query)
//   scores:  s[h,t]   = sum_{j<rk_t} Ck[t,j] q'[h,j]                       (kernel attn_partial)
//   softmax: online, base 2, fp32, per split of the token axis
//   sum:     u[h,j]   = sum_{t: rv_t>j} p[h,t] Cv[t,j]
//   merge:   splits combined with their (max, sum) pairs                   (kernel merge_expand)
//   expand:  out[h,i] = sum_j u[h,j] Bv[j, h*d+i]
//
// attn_partial is the HBM-bound kernel.  One workgroup (4 waves, one per SIMD) owns one
// (sequence, token split).  Coefficient tiles of 32 tokens travel HBM -> LDS with
// direct-to-LDS loads through a 3-deep ring (K tile, V tile, K tile, ...), two stages in
// flight while one is consumed, so no VGPR is spent on staging.  Every wave serves all
// heads on a quarter of the rank axis, so each tile byte is read from LDS exactly once:
//   S^T[t,h]  = Ck_tile[t,:] . q'^T      MFMA 16x16x32, A = tile rows (LDS), B = q' (VGPR);
//                                         the four waves' partial sums meet in LDS
//   U^T[j,h] += Cv_tile^T[j,t] . P^T     MFMA 16x16x32, A = register transpose of the tile
//                                         (v_perm), B = P (the S^T accumulator layout is
//                                         exactly the B-operand layout, so P never leaves
//                                         registers)
// For bf16 storage q' and P are split into hi+lo bf16 pairs (two MFMAs) so that the
// operand rounding stays far inside the 2e-3 tolerance; fp16 needs no split.
#include "ap_common.hpp"

namespace ap {
namespace {

constexpr int kTile = 32;        // tokens per tile
constexpr int kNBuf = 3;         // LDS ring depth
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <class Tag> struct Mfma;
template <> struct Mfma<F16Tag> {
  static __device__ __forceinline__ f32x4_t run(u32x4_t a, u32x4_t b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                  __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
};
template <> struct Mfma<BF16Tag> {
  static __device__ __forceinline__ f32x4_t run(u32x4_t a, u32x4_t b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};

__device__ __forceinline__ void dma16(const void* gsrc, void* lds_uniform) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_uniform, 16, 0, 0);
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


// Two fp32 -> packed pair of 16-bit storage values, round to nearest even (hardware converts).
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 f16x2_t;
__device__ __forceinline__ uint32_t cvt_pack(float lo, float hi, BF16Tag) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ uint32_t cvt_pack(float lo, float hi, F16Tag) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}

// ------------------------------------------------------------------------------------------
// fold_query: grid (Hp, B), 256 threads.  Qp[b][0][h][j] = hi, Qp[b][1][h][j] = lo of
// sm_scale*log2e * (Bk[b][j, head h] . q[b,h]);  heads >= H are zero rows.
// ------------------------------------------------------------------------------------------
template <class Tag>
__global__ void __launch_bounds__(256)
fold_query(const uint16_t* __restrict__ q, const uint16_t* __restrict__ Bk, int64_t bstride,
           uint16_t* __restrict__ Qp, int H, int Hp, int d, int r, float scale) {
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  uint16_t* hi_row = Qp + (((size_t)b * 2 + 0) * Hp + h) * r;
  uint16_t* lo_row = Qp + (((size_t)b * 2 + 1) * Hp + h) * r;
  if (h >= H) {
    for (int j = tid; j < r; j += 256) { hi_row[j] = 0; lo_row[j] = 0; }
    return;
  }
  const int tpr = d >> 3;            // threads per basis row (power of two, <= 32)
  const int rows = 256 / tpr;
  const int rg = tid / tpr, cc = tid - rg * tpr;
  const size_t HD = (size_t)H * d;
  float qv[8];
  {
    const u32x4_t w = *(const u32x4_t*)(q + ((size_t)b * H + h) * d + cc * 8);
#pragma unroll
    for (int e = 0; e < 4; ++e) { qv[2 * e] = lo_to_f32(w[e], Tag{}); qv[2 * e + 1] = hi_to_f32(w[e], Tag{}); }
  }
  const uint16_t* Bb = Bk + (size_t)b * bstride + (size_t)h * d + cc * 8;
  for (int j0 = 0; j0 < r; j0 += rows) {
    const int j = j0 + rg;
    float acc = 0.f;
    if (j < r) {
      const u32x4_t w = *(const u32x4_t*)(Bb + (size_t)j * HD);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc = fmaf(lo_to_f32(w[e], Tag{}), qv[2 * e], acc);
        acc = fmaf(hi_to_f32(w[e], Tag{}), qv[2 * e + 1], acc);
      }
    }
    for (int o = tpr >> 1; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (cc == 0 && j < r) {
      uint16_t hi, lo;
      split_hi_lo<Tag>(acc * scale, hi, lo);
      hi_row[j] = hi;
      lo_row[j] = lo;
    }
  }
}


// ------------------------------------------------------------------------------------------
// tile kernels, fully unrolled for a compile-time number of steps (selected by a
// wave-uniform switch on the run-time rank, so the unrolled bodies carry no guards)
// ------------------------------------------------------------------------------------------
// Partial scores of one 32-token tile over this wave's NK_ score k-steps (32 columns
// each), for all MT head tiles.  The tile rows are read from LDS once and reused by
// every head tile.
template <class Tag, int MT, bool SPLIT, int NKW>
__device__ __forceinline__ void score_tile(int nk, const char* a0, const char* a1,
                                           const u32x4_t (&qhi)[NKW][MT],
                                           const u32x4_t (&qlo)[SPLIT ? NKW : 1][MT],
                                           f32x4_t (&s)[MT][2]) {
  u32x4_t A0 = *(const u32x4_t*)a0;
  u32x4_t A1 = *(const u32x4_t*)a1;
#pragma unroll
  for (int i = 0; i < NKW; ++i) {
    if (i >= nk) break;
    u32x4_t N0 = A0, N1 = A1;
    if (i + 1 < nk) {                      // prefetch the next k-step's rows
      N0 = *(const u32x4_t*)(a0 + (i + 1) * 256);
      N1 = *(const u32x4_t*)(a1 + (i + 1) * 256);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      s[mt][0] = Mfma<Tag>::run(A0, qhi[i][mt], s[mt][0]);
      s[mt][1] = Mfma<Tag>::run(A1, qhi[i][mt], s[mt][1]);
    }
    if (SPLIT) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        s[mt][0] = Mfma<Tag>::run(A0, qlo[i][mt], s[mt][0]);
        s[mt][1] = Mfma<Tag>::run(A1, qlo[i][mt], s[mt][1]);
      }
    }
    A0 = N0;
    A1 = N1;
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Weighted coefficient sum of one tile over NG_ 128-column groups.  In every group
// this wave owns the two columns 8n+2w, 8n+2w+1 of each lane's 8: one dword per row.
template <class Tag, int MT, bool SPLIT, int NGRP>
__device__ __forceinline__ void wsum_tile(int ng, const char* vb, int pitch, int r, int n,
                                          const u32x4_t (&Phi)[MT], const u32x4_t (&Plo)[MT],
                                          f32x4_t (&U)[NGRP][2][MT]) {
#pragma unroll
  for (int grp = 0; grp < NGRP; ++grp) {
    if (grp >= ng) break;
    uint32_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      v[e] = *(const uint32_t*)(vb + (16 * (e >> 2) + (e & 3)) * pitch + grp * 256);
    if (grp * 128 + n * 8 >= r) {   // half-filled last group
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = 0;
    }
    // 8x2 transpose of 16-bit elements: operand j holds column 8n+2w+j of the 8 tokens
    u32x4_t te, to;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      te[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], 0x05040100u);
      to[k] = __builtin_amdgcn_perm(v[2 * k + 1], v[2 * k], 0x07060302u);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      U[grp][0][mt] = Mfma<Tag>::run(te, Phi[mt], U[grp][0][mt]);
      U[grp][1][mt] = Mfma<Tag>::run(to, Phi[mt], U[grp][1][mt]);
    }
    if (SPLIT) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        U[grp][0][mt] = Mfma<Tag>::run(te, Plo[mt], U[grp][0][mt]);
        U[grp][1][mt] = Mfma<Tag>::run(to, Plo[mt], U[grp][1][mt]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// ------------------------------------------------------------------------------------------
// attn_partial
// ------------------------------------------------------------------------------------------
struct AttnParams {
  const uint16_t* Qp;   // [B][2][Hp][r]
  const uint16_t* Ck;   // [B][T_cap][r]
  const uint16_t* Cv;
  float* part_ml;       // [B][S][H][2]   (running max in log2 units, sum)
  float* part_U;        // [B][S][H][r]
  int T, T_cap, r, H, nsplit;
};

// Four waves, one per SIMD.  Every wave serves ALL heads (MT tiles of 16) on a quarter
// of the rank axis: score k-steps w, w+4, ... and, in every 128-column group of the
// weighted sum, two of each lane's eight columns.  The four partial score tiles are
// added through LDS once per token tile; each wave then runs the same softmax.
template <class Tag, int MT, int RMAX, bool SPLIT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
attn_partial(const AttnParams p) {
  constexpr int NKW = (RMAX / 32 + 3) / 4;         // score k-steps per wave
  constexpr int NGRP = (RMAX + 127) / 128;         // 128-column groups
  constexpr int MAXBLK = (RMAX / 8 + 1 + 1) / 2;   // 1 KiB blocks per stage, padded rows
  constexpr int NSLOT = (MAXBLK + 3) / 4;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, n = lane & 15, g = lane >> 4;
  const int b = blockIdx.y, s = blockIdx.x;
  const int r = p.r, T = p.T, H = p.H;
  constexpr int Hp = MT * 16;

  // ---- stage geometry: 32 rows of (cpr+1) 16-byte chunks (one pad chunk per row keeps
  //      8 consecutive rows on 8 different bank groups for the row-strided operand reads)
  const int cpr = r >> 3;
  const int pitch = (cpr + 1) * 16;
  const int tot_chunks = kTile * (cpr + 1);
  const int nblk = (tot_chunks + 63) >> 6;
  const int stage_bytes = nblk * 1024;
  f32x4_t* xchg = (f32x4_t*)(smem + kNBuf * stage_bytes);   // [4 waves][2*MT][64 lanes]

  // ---- this wave's share of a stage: blocks w, w+4, ...; per lane (row, byte offset)
  uint32_t slot[NSLOT];
  int n_issue = 0;
#pragma unroll
  for (int k = 0; k < NSLOT; ++k) {
    const int blk = w + 4 * k;
    slot[k] = 0;
    if (blk < nblk) {
      ++n_issue;
      const int L = blk * 64 + lane;
      int row = L / (cpr + 1);
      int c = L - row * (cpr + 1);
      if (L >= tot_chunks) { row = 0; c = 0; }   // tail of the last block: harmless duplicate
      if (c == cpr) c = 0;                        // pad chunk: harmless duplicate
      slot[k] = ((uint32_t)row << 16) | (uint32_t)(c * 16);
    }
  }

  // ---- token tiles of this split
  const int ntiles = (T + kTile - 1) / kTile;
  const int t_lo = (int)(((int64_t)s * ntiles) / p.nsplit);
  const int t_hi = (int)(((int64_t)(s + 1) * ntiles) / p.nsplit);
  const int nq = 2 * (t_hi - t_lo);

  const char* Ck_b = (const char*)(p.Ck + (size_t)b * p.T_cap * r);
  const char* Cv_b = (const char*)(p.Cv + (size_t)b * p.T_cap * r);
  const uint32_t row_bytes = (uint32_t)r * 2u;

  auto issue = [&](int q) {
    const int tok0 = (t_lo + (q >> 1)) * kTile;
    const char* src = (q & 1) ? Cv_b : Ck_b;
    char* dst = smem + (q % kNBuf) * stage_bytes;
#pragma unroll
    for (int k = 0; k < NSLOT; ++k) {
      const int blk = w + 4 * k;
      if (blk < nblk) {
        int tok = tok0 + (int)(slot[k] >> 16);
        tok = tok < T ? tok : T - 1;
        const char* ga = src + (size_t)tok * row_bytes + (slot[k] & 0xffffu);
        dma16(ga, dst + blk * 1024);
      }
    }
  };

  if (nq > 0) issue(0);
  if (nq > 1) issue(1);

  // ---- this wave's quarter
  const int nks = r >> 5;                               // all score k-steps
  const int my_nks = nks > w ? (nks - w + 3) >> 2 : 0;  // k-steps w, w+4, ...
  const int ngrp = (r + 127) >> 7;

  // ---- q' operands (B operand of the score MFMA): lane (h=n, g) holds columns 32ks+8g..+7
  u32x4_t qhi[NKW][MT];
  u32x4_t qlo[SPLIT ? NKW : 1][MT];
#pragma unroll
  for (int i = 0; i < NKW; ++i)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      u32x4_t z = {0, 0, 0, 0};
      qhi[i][mt] = z;
      if (SPLIT) qlo[i][mt] = z;
      if (i < my_nks) {
        const uint16_t* qrow =
            p.Qp + (((size_t)b * 2) * Hp + (mt * 16 + n)) * r + (w + 4 * i) * 32 + g * 8;
        qhi[i][mt] = *(const u32x4_t*)qrow;
        if (SPLIT) qlo[i][mt] = *(const u32x4_t*)(qrow + (size_t)Hp * r);
      }
    }

  f32x4_t U[NGRP][2][MT];
#pragma unroll
  for (int grp = 0; grp < NGRP; ++grp)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) { f32x4_t z = {0.f, 0.f, 0.f, 0.f}; U[grp][j][mt] = z; }
  float m_run[MT], l_run[MT];   // running max of head 16mt+n; this lane's share of the sum
  u32x4_t Phi[MT], Plo[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    m_run[mt] = -INFINITY;
    l_run[mt] = 0.f;
    u32x4_t z = {0, 0, 0, 0};
    Phi[mt] = z;
    Plo[mt] = z;
  }

  for (int q = 0; q < nq; ++q) {
    // loads of stage q must have landed; those of stage q+1 may stay in flight
    wait_vmcnt(q + 1 < nq ? n_issue : 0);
    wg_barrier();   // stage q complete for every wave; everyone is done with stage q-1
    if (q + 2 < nq) issue(q + 2);
    const char* buf = smem + (q % kNBuf) * stage_bytes;
    if ((q & 1) == 0) {
      // ================= scores + online softmax for tile q/2 =================
      const int tok0 = (t_lo + (q >> 1)) * kTile;
      const char* a0 = buf + n * pitch + g * 16 + w * 64;
      const char* a1 = a0 + 16 * pitch;
      f32x4_t sp[MT][2];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) { f32x4_t z = {0.f, 0.f, 0.f, 0.f}; sp[mt][0] = z; sp[mt][1] = z; }
      score_tile<Tag, MT, SPLIT, NKW>(my_nks, a0, a1, qhi, qlo, sp);
      // add the four waves' partial scores in a fixed order, so that every wave
      // carries bit-identical maxima, weights and sums from here on
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        xchg[(w * 2 * MT + 2 * mt + 0) * 64 + lane] = sp[mt][0];
        xchg[(w * 2 * MT + 2 * mt + 1) * 64 + lane] = sp[mt][1];
      }
      wg_barrier();
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        f32x4_t t0 = xchg[(0 * 2 * MT + 2 * mt + 0) * 64 + lane];
        f32x4_t t1 = xchg[(0 * 2 * MT + 2 * mt + 1) * 64 + lane];
#pragma unroll
        for (int ww = 1; ww < 4; ++ww) {
          t0 += xchg[(ww * 2 * MT + 2 * mt + 0) * 64 + lane];
          t1 += xchg[(ww * 2 * MT + 2 * mt + 1) * 64 + lane];
        }
        float sc[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) { sc[i] = t0[i]; sc[4 + i] = t1[i]; }
        // lane (h=n, g) holds tokens tok0 + 16*tt + 4*g + i
        float tmax = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int tok = tok0 + 16 * (e >> 2) + 4 * g + (e & 3);
          if (tok >= T) sc[e] = -INFINITY;
          tmax = fmaxf(tmax, sc[e]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run[mt], tmax);   // finite: every tile holds a valid token
        const float alpha = fast_exp2(m_run[mt] - m_new);
        m_run[mt] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float p0 = fast_exp2(sc[2 * k] - m_new), p1 = fast_exp2(sc[2 * k + 1] - m_new);
          const uint32_t hi = cvt_pack(p0, p1, Tag{});
          float k0 = lo_to_f32(hi, Tag{}), k1 = hi_to_f32(hi, Tag{});
          Phi[mt][k] = hi;
          if (SPLIT) {
            const uint32_t lo = cvt_pack(p0 - k0, p1 - k1, Tag{});
            Plo[mt][k] = lo;
            k0 += lo_to_f32(lo, Tag{});
            k1 += hi_to_f32(lo, Tag{});
          }
          psum += k0 + k1;                             // the sum uses the values the MFMA will see
        }
        l_run[mt] = l_run[mt] * alpha + psum;
#pragma unroll
          for (int grp = 0; grp < NGRP; ++grp) {
            U[grp][0][mt] *= alpha;
            U[grp][1][mt] *= alpha;
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      // ================= weighted coefficient sum for tile q/2 =================
      const char* vb = buf + (4 * g) * pitch + n * 16 + w * 4;
      wsum_tile<Tag, MT, SPLIT, NGRP>(ngrp, vb, pitch, r, n, Phi, Plo, U);
    }
  }

  // ---- epilogue: (m, l) and U of this split.  U[grp][j][mt][i] is element
  //      (head 16mt+n, column 128grp + 32g + 8i + 2w + j); one head tile at a time is
  //      transposed through LDS so that rows leave coalesced.
  const size_t pbase = ((size_t)b * p.nsplit + s) * H;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float l_tot = l_run[mt];
    l_tot += __shfl_xor(l_tot, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (w == 0 && g == 0 && mt * 16 + n < H) {
      p.part_ml[(pbase + mt * 16 + n) * 2 + 0] = m_run[mt];
      p.part_ml[(pbase + mt * 16 + n) * 2 + 1] = l_tot;
    }
  }
  float* ul = (float*)smem;                       // [16][r+1]
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    wg_barrier();                                 // ring / previous head tile no longer read
#pragma unroll
    for (int grp = 0; grp < NGRP; ++grp)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int col = grp * 128 + g * 32 + i * 8 + 2 * w + j;
          if (col < r) ul[n * (r + 1) + col] = U[grp][j][mt][i];
        }
    wg_barrier();
    for (int hh = w; hh < 16 && mt * 16 + hh < H; hh += 4) {
      float* dst = p.part_U + (pbase + mt * 16 + hh) * r;
      for (int j = lane; j < r; j += 64) dst[j] = ul[hh * (r + 1) + j];
    }
  }
}

// ------------------------------------------------------------------------------------------
// merge_expand: grid (H, B), 256 threads.  Combine the splits of head h, then
// out[b,h,:] = u . Bv[b][:, head h].
// ------------------------------------------------------------------------------------------
template <class Tag, bool OUT_F32>
__global__ void __launch_bounds__(256)
merge_expand(const float* __restrict__ part_ml, const float* __restrict__ part_U,
             const uint16_t* __restrict__ Bv, int64_t bstride, void* __restrict__ out,
             float* __restrict__ lse, int H, int d, int r, int nsplit) {
  extern __shared__ __attribute__((aligned(16))) char smem_me[];
  float* ustar = (float*)smem_me;          // [r]
  float* red = ustar + r;                  // [rows][d]
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const size_t pb = (size_t)b * nsplit * H + h;    // + s*H
  float mstar = -INFINITY;
  for (int s = 0; s < nsplit; ++s) mstar = fmaxf(mstar, part_ml[(pb + (size_t)s * H) * 2]);
  float L = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float ms = part_ml[(pb + (size_t)s * H) * 2];
    const float ls = part_ml[(pb + (size_t)s * H) * 2 + 1];
    L += ls * fast_exp2(ms - mstar);
  }
  const float invL = 1.0f / L;
  for (int j = tid; j < r; j += 256) {
    float acc = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const float ws = fast_exp2(part_ml[(pb + (size_t)s * H) * 2] - mstar);
      acc = fmaf(ws, part_U[(pb + (size_t)s * H) * r + j], acc);
    }
    ustar[j] = acc * invL;
  }
  __syncthreads();
  const int tpr = d >> 3, rows = 256 / tpr;
  const int rg = tid / tpr, cc = tid - rg * tpr;
  const size_t HD = (size_t)H * d;
  const uint16_t* Bb = Bv + (size_t)b * bstride + (size_t)h * d + cc * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int j = rg; j < r; j += rows) {
    const u32x4_t wv = *(const u32x4_t*)(Bb + (size_t)j * HD);
    const float u = ustar[j];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc[2 * e] = fmaf(u, lo_to_f32(wv[e], Tag{}), acc[2 * e]);
      acc[2 * e + 1] = fmaf(u, hi_to_f32(wv[e], Tag{}), acc[2 * e + 1]);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rg * d + cc * 8 + e] = acc[e];
  __syncthreads();
  for (int i = tid; i < d; i += 256) {
    float sum = 0.f;
    for (int k = 0; k < rows; ++k) sum += red[k * d + i];
    if (OUT_F32) ((float*)out)[((size_t)b * H + h) * d + i] = sum;
    else ((uint16_t*)out)[((size_t)b * H + h) * d + i] = f32_to_bits(sum, Tag{});
  }
  if (tid == 0 && lse) lse[(size_t)b * H + h] = (mstar + log2f(L)) * kLn2;
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
int device_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      cus = v;
    else
      cus = 256;
  }
  return cus;
}

// Splits of the token axis: enough workgroups to cover every CU once, never finer
// than one 32-token tile.  The count does not depend on the device, so the workspace
// query needs no GPU.
int choose_nsplit(int B, int T) {
  const int ntiles = (T + kTile - 1) / kTile;
  int s = (256 + B - 1) / B;
  if (s > ntiles) s = ntiles;
  if (s < 1) s = 1;
  return s;
}

struct WsLayout {
  size_t qp, ml, u, total;
};
WsLayout ws_layout(int B, int H, int T, int r) {
  const int Hp = (H + 15) / 16 * 16;
  const int S = choose_nsplit(B, T);
  WsLayout w;
  w.qp = 0;
  size_t off = round_up((size_t)B * 2 * Hp * r * 2, 256);
  w.ml = off;
  off += round_up((size_t)B * S * H * 2 * 4, 256);
  w.u = off;
  off += round_up((size_t)B * S * H * r * 4, 256);
  w.total = off;
  return w;
}

template <class Tag, int MT, int RMAX, bool SPLIT>
ap_status launch_attn(const AttnParams& p, int B, hipStream_t stream) {
  const int cpr = p.r / 8;
  const int nblk = (kTile * (cpr + 1) + 63) / 64;
  size_t ring = (size_t)kNBuf * nblk * 1024 + (size_t)4 * 2 * MT * 64 * 16;
  size_t epi = (size_t)16 * (p.r + 1) * 4;
  size_t lds = ring > epi ? ring : epi;
  AP_REQUIRE(lds <= 160 * 1024, AP_ERR_UNSUPPORTED, "ap_decode_attn: LDS need %zu > 160 KiB", lds);
  auto kern = attn_partial<Tag, MT, RMAX, SPLIT>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       160 * 1024);
    if (e != hipSuccess) {
      set_error("hipFuncSetAttribute: %s", hipGetErrorString(e));
      return AP_ERR_HIP;
    }
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(p.nsplit, B), dim3(256), lds, stream, p);
  return AP_OK;
}

template <class Tag, bool SPLIT>
ap_status dispatch_attn(const AttnParams& p, int B, hipStream_t stream) {
  const int nw = (p.H + 15) / 16;
#define AP_CASE(NWV)                                                              \
  case NWV:                                                                       \
    return p.r <= 256 ? launch_attn<Tag, NWV, 256, SPLIT>(p, B, stream)           \
                      : launch_attn<Tag, NWV, 640, SPLIT>(p, B, stream);
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
  const int S = choose_nsplit(a.B, a.T);
  const WsLayout wl = ws_layout(a.B, a.H, a.T, a.r);
  char* ws = (char*)a.workspace;
  uint16_t* Qp = (uint16_t*)(ws + wl.qp);
  float* ml = (float*)(ws + wl.ml);
  float* U = (float*)(ws + wl.u);
  hipLaunchKernelGGL(fold_query<Tag>, dim3(Hp, a.B), dim3(256), 0, a.stream, (const uint16_t*)a.q,
                     (const uint16_t*)a.Bk, a.basis_batch_stride, Qp, a.H, Hp, a.d, a.r,
                     a.sm_scale * kLog2e);
  AttnParams p{Qp, (const uint16_t*)a.Ck, (const uint16_t*)a.Cv, ml, U, a.T, a.T_cap, a.r, a.H, S};
  ap_status st = dispatch_attn<Tag, SPLIT>(p, a.B, a.stream);
  if (st != AP_OK) return st;
  const int rows = 256 / (a.d / 8);
  const size_t lds = ((size_t)a.r + (size_t)rows * a.d) * 4;
  if (a.dt_out == AP_F32)
    hipLaunchKernelGGL((merge_expand<Tag, true>), dim3(a.H, a.B), dim3(256), lds, a.stream, ml, U,
                       (const uint16_t*)a.Bv, a.basis_batch_stride, a.out, a.lse, a.H, a.d, a.r, S);
  else
    hipLaunchKernelGGL((merge_expand<Tag, false>), dim3(a.H, a.B), dim3(256), lds, a.stream, ml, U,
                       (const uint16_t*)a.Bv, a.basis_batch_stride, a.out, a.lse, a.H, a.d, a.r, S);
  return check_launch("ap_decode_attn");
}

}  // namespace

size_t decode_mfma_workspace(int B, int H, int d, int T, int r, ap_dtype dt) {
  (void)d;
  (void)dt;
  return ws_layout(B, H, T, r).total;
}

ap_status launch_decode_mfma(const DecodeArgs& a) {
  AP_REQUIRE(a.B <= 65535, AP_ERR_UNSUPPORTED, "ap_decode_attn: B must be <= 65535");
  AP_REQUIRE(a.dt_coef != AP_I8, AP_ERR_UNSUPPORTED, "ap_decode_attn: int8 coefficients not built yet");
  AP_REQUIRE(!a.rank_k && !a.rank_v, AP_ERR_UNSUPPORTED, "ap_decode_attn: ragged ranks not built yet");
  return a.dt == AP_F16 ? run_decode<F16Tag, false>(a) : run_decode<BF16Tag, true>(a);
}

}  // namespace ap
