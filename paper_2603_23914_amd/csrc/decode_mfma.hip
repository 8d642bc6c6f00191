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
// attn_partial is the HBM-bound kernel.  One workgroup owns one (sequence, token
// split); wave w owns heads 16w..16w+15 for ALL r columns.  Coefficient tiles of 32
// tokens travel HBM -> LDS with direct-to-LDS loads through a 3-deep ring (K tile,
// V tile, K tile, ...), two stages in flight while one is consumed, so no VGPR is
// spent on staging.  Every wave reads the whole tile from LDS:
//   S^T[t,h]  = Ck_tile[t,:] . q'^T      MFMA 16x16x32, A = tile rows (LDS), B = q' (VGPR)
//   U^T[j,h] += Cv_tile^T[j,t] . P^T     MFMA 16x16x32, A = 8x8 register transpose of the
//                                         tile (v_perm), B = P (the S^T accumulator layout
//                                         is exactly the B-operand layout, so P never
//                                         leaves registers)
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
// Partial scores of one 32-token tile over NKS_*32 coefficient columns.
template <class Tag, bool SPLIT, int NKS_>
__device__ __forceinline__ void score_tile(const char* a0, const char* a1, const u32x4_t* qhi,
                                           const u32x4_t* qlo, f32x4_t& s0, f32x4_t& s1) {
  f32x4_t sh0 = {0.f, 0.f, 0.f, 0.f}, sh1 = sh0, sl0 = sh0, sl1 = sh0;
#pragma unroll
  for (int ks = 0; ks < NKS_; ++ks) {
    const u32x4_t A0 = *(const u32x4_t*)(a0 + ks * 64);
    const u32x4_t A1 = *(const u32x4_t*)(a1 + ks * 64);
    sh0 = Mfma<Tag>::run(A0, qhi[ks], sh0);
    sh1 = Mfma<Tag>::run(A1, qhi[ks], sh1);
    if (SPLIT) {
      sl0 = Mfma<Tag>::run(A0, qlo[ks], sl0);
      sl1 = Mfma<Tag>::run(A1, qlo[ks], sl1);
    }
  }
  s0 = SPLIT ? sh0 + sl0 : sh0;
  s1 = SPLIT ? sh1 + sl1 : sh1;
}

// One 128-column group of the weighted coefficient sum: Ug[c] += Cv_tile^T . P.
// `lane_valid` is false for lanes whose 8 columns lie at or beyond the rank.
template <class Tag, bool SPLIT>
__device__ __forceinline__ void wsum_group(const char* vb, int pitch, bool lane_valid,
                                           const u32x4_t& Phi, const u32x4_t& Plo,
                                           f32x4_t (&Ug)[8]) {
  u32x4_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e)
    v[e] = *(const u32x4_t*)(vb + (16 * (e >> 2) + (e & 3)) * pitch);
  if (!lane_valid) {
#pragma unroll
    for (int e = 0; e < 8; ++e) { u32x4_t z = {0, 0, 0, 0}; v[e] = z; }
  }
  // 8x8 transpose of 16-bit elements: operand c holds column 8n+c of the 8 tokens
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    u32x4_t t;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      t[k] = __builtin_amdgcn_perm(v[2 * k + 1][c >> 1], v[2 * k][c >> 1],
                                   (c & 1) ? 0x07060302u : 0x05040100u);
    Ug[c] = Mfma<Tag>::run(t, Phi, Ug[c]);
    if (SPLIT) Ug[c] = Mfma<Tag>::run(t, Plo, Ug[c]);
  }
}

template <class Tag, bool SPLIT, int NG, int NG_>
__device__ __forceinline__ void wsum_tile(const char* vb, int pitch, int cols_left, int n,
                                          const u32x4_t& Phi, const u32x4_t& Plo,
                                          f32x4_t (&U)[NG][8]) {
#pragma unroll
  for (int gi = 0; gi < NG_; ++gi) {
    const bool valid = gi * 128 + n * 8 < cols_left;
    wsum_group<Tag, SPLIT>(vb + gi * 256, pitch, valid, Phi, Plo, U[gi]);
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

// Waves come in pairs: wave 2*mt+half owns heads 16mt..16mt+15 and one half of the r
// columns (half of the score k-steps, half of the 128-column groups of the weighted
// sum).  The two halves of a pair add their partial scores through LDS once per tile.
template <class Tag, int NW, int RMAX, bool SPLIT>
__global__ void __launch_bounds__(NW * 128) __attribute__((amdgpu_waves_per_eu(1, 2)))
attn_partial(const AttnParams p) {
  constexpr int NWV = 2 * NW;                      // waves per workgroup
  constexpr int NKSH = RMAX / 64;                  // score k-steps (32 columns) per half
  constexpr int NCB = (RMAX + 127) / 128;          // 128-column groups in all
  constexpr int NG = (NCB + 1) / 2;                // groups per half (first half gets the odd one)
  constexpr int MAXBLK = (RMAX / 8 + 1 + 1) / 2;   // 1 KiB blocks per stage, padded rows
  constexpr int NSLOT = (MAXBLK + NWV - 1) / NWV;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int tid = threadIdx.x;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mt = wv >> 1, half = wv & 1;
  const int lane = tid & 63, n = lane & 15, g = lane >> 4;
  const int b = blockIdx.y, s = blockIdx.x;
  const int r = p.r, T = p.T, H = p.H;
  const int Hp = NW * 16;

  // ---- stage geometry: 32 rows of (cpr+1) 16-byte chunks (one pad chunk per row keeps
  //      8 consecutive rows on 8 different bank groups for the row-strided operand reads)
  const int cpr = r >> 3;
  const int pitch = (cpr + 1) * 16;
  const int tot_chunks = kTile * (cpr + 1);
  const int nblk = (tot_chunks + 63) >> 6;
  const int stage_bytes = nblk * 1024;
  char* xchg = smem + kNBuf * stage_bytes;          // [NWV][64 lanes][32 B] partial scores

  // ---- this wave's share of a stage: blocks wv, wv+NWV, ...; per lane (row, byte offset)
  uint32_t slot[NSLOT];
  int n_issue = 0;
#pragma unroll
  for (int k = 0; k < NSLOT; ++k) {
    const int blk = wv + NWV * k;
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
      const int blk = wv + NWV * k;
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

  // ---- this wave's halves
  const int nks = r >> 5;                // all score k-steps (even: r % 64 == 0)
  const int my_nks = nks >> 1;
  const int ks0 = half * my_nks;
  const int ncb = (r + 127) >> 7;
  const int ng0 = (ncb + 1) >> 1;
  const int cb0 = half * ng0;
  const int my_ng = half ? ncb - ng0 : ng0;
  const int cols_left = r - cb0 * 128;   // columns from my first group to the rank

  // ---- q' operands (B operand of the score MFMA): lane (h=n, g) holds columns 32ks+8g..+7
  u32x4_t qhi[NKSH];
  u32x4_t qlo[SPLIT ? NKSH : 1];
  {
    const uint16_t* qrow = p.Qp + (((size_t)b * 2) * Hp + (mt * 16 + n)) * r + ks0 * 32 + g * 8;
#pragma unroll
    for (int i = 0; i < NKSH; ++i) {
      u32x4_t z = {0, 0, 0, 0};
      qhi[i] = z;
      if (SPLIT) qlo[i] = z;
      if (i < my_nks) {
        qhi[i] = *(const u32x4_t*)(qrow + i * 32);
        if (SPLIT) qlo[i] = *(const u32x4_t*)(qrow + (size_t)Hp * r + i * 32);
      }
    }
  }

  f32x4_t U[NG][8];
#pragma unroll
  for (int gi = 0; gi < NG; ++gi)
#pragma unroll
    for (int c = 0; c < 8; ++c) { f32x4_t z = {0.f, 0.f, 0.f, 0.f}; U[gi][c] = z; }
  float m_run = -INFINITY;   // running max of head n (same in the 4 lanes that share n)
  float l_run = 0.f;         // this lane's share of the running sum
  u32x4_t Phi = {0, 0, 0, 0}, Plo = {0, 0, 0, 0};

  f32x4_t* my_x = (f32x4_t*)(xchg + (wv * 64 + lane) * 32);
  const f32x4_t* peer_x = (const f32x4_t*)(xchg + ((wv ^ 1) * 64 + lane) * 32);

  for (int q = 0; q < nq; ++q) {
    // loads of stage q must have landed; those of stage q+1 may stay in flight
    wait_vmcnt(q + 1 < nq ? n_issue : 0);
    wg_barrier();   // stage q complete for every wave; everyone is done with stage q-1
    if (q + 2 < nq) issue(q + 2);
    const char* buf = smem + (q % kNBuf) * stage_bytes;
    if ((q & 1) == 0) {
      // ================= scores + online softmax for tile q/2 =================
      const int tok0 = (t_lo + (q >> 1)) * kTile;
      const char* a0 = buf + n * pitch + g * 16 + ks0 * 64;
      const char* a1 = a0 + 16 * pitch;
      f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
#define AP_SCORE_CASE(K)                                                             \
  case K:                                                                            \
    if constexpr (K <= NKSH) score_tile<Tag, SPLIT, K>(a0, a1, qhi, qlo, s0, s1);    \
    break;
      switch (my_nks) {
        AP_SCORE_CASE(1) AP_SCORE_CASE(2) AP_SCORE_CASE(3) AP_SCORE_CASE(4) AP_SCORE_CASE(5)
        AP_SCORE_CASE(6) AP_SCORE_CASE(7) AP_SCORE_CASE(8) AP_SCORE_CASE(9) AP_SCORE_CASE(10)
        default: break;
      }
#undef AP_SCORE_CASE
      // add the other half's partial scores (a+b == b+a bit for bit, so both waves of
      // the pair carry identical maxima, weights and sums from here on)
      my_x[0] = s0;
      my_x[1] = s1;
      wg_barrier();
      const f32x4_t o0 = peer_x[0], o1 = peer_x[1];
      float sc[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) { sc[i] = s0[i] + o0[i]; sc[4 + i] = s1[i] + o1[i]; }
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
      const float m_new = fmaxf(m_run, tmax);     // finite: every tile holds a valid token
      const float alpha = fast_exp2(m_run - m_new);
      m_run = m_new;
      float psum = 0.f;
      uint16_t ph[8], pl[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pe = fast_exp2(sc[e] - m_new);
        ph[e] = f32_to_bits(pe, Tag{});
        float kept = bits_to_f32(ph[e], Tag{});
        if (SPLIT) {
          pl[e] = f32_to_bits(pe - kept, Tag{});
          kept += bits_to_f32(pl[e], Tag{});
        }
        psum += kept;                              // the sum uses the values the MFMA will see
      }
      l_run = l_run * alpha + psum;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        Phi[k] = (uint32_t)ph[2 * k] | ((uint32_t)ph[2 * k + 1] << 16);
        if (SPLIT) Plo[k] = (uint32_t)pl[2 * k] | ((uint32_t)pl[2 * k + 1] << 16);
      }
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int gi = 0; gi < NG; ++gi)
#pragma unroll
          for (int c = 0; c < 8; ++c) U[gi][c] *= alpha;
      }
    } else {
      // ================= weighted coefficient sum for tile q/2 =================
      const char* vb = buf + (4 * g) * pitch + n * 16 + cb0 * 256;
#define AP_WSUM_CASE(K)                                                                         \
  case K:                                                                                       \
    if constexpr (K <= NG) wsum_tile<Tag, SPLIT, NG, K>(vb, pitch, cols_left, n, Phi, Plo, U);   \
    break;
      switch (my_ng) {
        AP_WSUM_CASE(1) AP_WSUM_CASE(2) AP_WSUM_CASE(3)
        default: break;
      }
#undef AP_WSUM_CASE
    }
  }

  // ---- epilogue: (m, l) and U of this split.  U[gi][c][i] is element
  //      (head 16mt+n, column 128(cb0+gi) + 32g + 8i + c); transpose through LDS so that
  //      rows leave coalesced.
  float l_tot = l_run;
  l_tot += __shfl_xor(l_tot, 16);
  l_tot += __shfl_xor(l_tot, 32);
  const size_t pbase = ((size_t)b * p.nsplit + s) * H;
  if (half == 0 && g == 0 && mt * 16 + n < H) {
    p.part_ml[(pbase + mt * 16 + n) * 2 + 0] = m_run;
    p.part_ml[(pbase + mt * 16 + n) * 2 + 1] = l_tot;
  }
  wg_barrier();                                   // ring no longer read by anyone
  float* ul = (float*)smem;                       // [Hp][r+1]
#pragma unroll
  for (int gi = 0; gi < NG; ++gi)
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int col = (cb0 + gi) * 128 + g * 32 + i * 8 + c;
        if (gi < my_ng && col < r) ul[(mt * 16 + n) * (r + 1) + col] = U[gi][c][i];
      }
  wg_barrier();
  for (int hh = wv; hh < H; hh += NWV) {
    float* dst = p.part_U + (pbase + hh) * r;
    for (int j = lane; j < r; j += 64) dst[j] = ul[hh * (r + 1) + j];
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

template <class Tag, int NW, int RMAX, bool SPLIT>
ap_status launch_attn(const AttnParams& p, int B, hipStream_t stream) {
  const int cpr = p.r / 8;
  const int nblk = (kTile * (cpr + 1) + 63) / 64;
  size_t ring = (size_t)kNBuf * nblk * 1024 + (size_t)2 * NW * 64 * 32;
  size_t epi = (size_t)NW * 16 * (p.r + 1) * 4;
  size_t lds = ring > epi ? ring : epi;
  AP_REQUIRE(lds <= 160 * 1024, AP_ERR_UNSUPPORTED, "ap_decode_attn: LDS need %zu > 160 KiB", lds);
  auto kern = attn_partial<Tag, NW, RMAX, SPLIT>;
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
  hipLaunchKernelGGL(kern, dim3(p.nsplit, B), dim3(NW * 128), lds, stream, p);
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
