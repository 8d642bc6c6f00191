// Key-only compression on the matrix cores (head width 128, key rank up to 128, up to 16 query
// heads per key/value head): the shape of the paper's text-domain experiment (appendix "Analysis
// of Textual Token Compression": keys compressed to R_k = 64, values kept).
//
// The flash-decode kernels on the vector ALU spend H*d fused multiply-adds per token on the value
// sum alone and are bound by that arithmetic once the keys are this small.  Here a wave takes a
// tile of 32 tokens of ONE key/value head and all the query heads that share it:
//   scores   S[token, head] = C_k[token, :r] . q'[head, :r]   MFMA 16x16x32, coefficient rows
//            straight from global memory into the A operand (16 rows x 64 bytes per load),
//            the folded queries (hi + lo halves for bf16) resident as B operands;
//   softmax  the MFMA result already has the layout of the next product's B operand (lane
//            (head, g) holds tokens 4g..4g+3 and 16+4g..16+4g+3), so the weights never leave
//            the registers: one maximum over the four lanes of a head, exponentials, hi + lo
//            split to the storage type;
//   values   O^T[column, head] += V^T[column, token] . P^T[token, head]: the wave's value tile
//            (32 rows x 256 bytes) goes through a private LDS region with a padded pitch, is
//            read back as dwords of eight token rows and transposed with byte permutes, as the
//            coefficient sums of the two-sided kernel are.
// The four waves of a workgroup take every fourth tile of the workgroup's token range and keep
// separate running (maximum, sum, output); every wave writes a normalised partial result, and
// merge_parts joins the 4 S parts of a head.
#include "ap_common.hpp"
#include "lane_ops.hpp"
#include "mfma_ops.hpp"
#include <type_traits>

namespace ap {
namespace {

constexpr int kTok = 32;           // tokens per tile
constexpr int kPitch = 272;        // bytes per value row in LDS: 256 + 16, so that the rows a
                                   // lane group reads fall on different banks
constexpr int kWaves = 4;

// grid: 8 * H_kv * ceil(B S / 8) workgroups of 256 threads.  Workgroup id -> (pair p = b S + su,
// key/value head): the H_kv workgroups of a pair follow each other on ONE XCD (ids 8 apart),
// so the pair's coefficient rows, which every head reads, are fetched from HBM once.
template <class Tag, int NKS>
__global__ void __launch_bounds__(256)
keyonly_mfma(const uint16_t* __restrict__ Qp, const uint16_t* __restrict__ Ck,
             const uint16_t* __restrict__ V, float* __restrict__ out_part, float* __restrict__ lse_part,
             int B, int H, int QG, int T, int T_cap, int r, int S, int per) {
  __shared__ __attribute__((aligned(16))) char vt[kWaves][kTok * kPitch];
  // bf16 carries 8 significant bits: folded queries and weights go to the matrix cores as hi + lo
  // pairs; fp16 (11 bits) needs no second half
  constexpr bool SPLIT = std::is_same<Tag, BF16Tag>::value;
  const int Hkv = H / QG;
  const int id = blockIdx.x, k = id >> 3;
  const int kvh = k % Hkv, p = (k / Hkv) * 8 + (id & 7);
  if (p >= B * S) return;
  const int b = p / S, su = p - b * S;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63, n = lane & 15, g = lane >> 4;
  const int h0 = kvh * QG;
  const size_t HD = (size_t)Hkv * 128;

  // folded queries of head h0 + n (zero beyond the heads of the group and beyond the rank)
  u32x4_t qh[NKS], ql[SPLIT ? NKS : 1];
  uint32_t koff[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const int col = ks * 32 + g * 8;
    const u32x4_t z = {0, 0, 0, 0};
    qh[ks] = z;
    if (SPLIT) ql[ks] = z;
    koff[ks] = col < r ? (uint32_t)col : 0u;          // columns beyond the rank re-read column 0
    if (n < QG && col < r) {
      const uint16_t* qp = Qp + (((size_t)b * 2) * H + h0 + n) * r + col;
      qh[ks] = *(const u32x4_t*)qp;
      if (SPLIT) ql[ks] = *(const u32x4_t*)(qp + (size_t)H * r);
    }
  }
  const uint16_t* Cb = Ck + (size_t)b * T_cap * r;
  const uint16_t* Vb = V + (size_t)b * T_cap * HD + (size_t)kvh * 128 + n * 8;
  const int t0 = su * per;
  int t1 = t0 + per;
  t1 = t1 < T ? t1 : T;
  const int ntiles = t1 > t0 ? (t1 - t0 + kTok - 1) / kTok : 0;

  // tile t of the split: coefficient rows 16 tt + n as A operands, value chunks (row 4 k2 + g,
  // 16-byte column n); rows beyond the range repeat its last row (masked in the softmax)
  u32x4_t A[NKS][2], Vr[8];
  auto load_tile = [&](int t) {
    const int base = t0 + t * kTok;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      int row = base + 16 * tt + n;
      row = row < t1 ? row : t1 - 1;
      const uint16_t* crow = Cb + (size_t)row * r;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) A[ks][tt] = *(const u32x4_t*)(crow + koff[ks]);
    }
#pragma unroll
    for (int k2 = 0; k2 < 8; ++k2) {
      int row = base + 4 * k2 + g;
      row = row < t1 ? row : t1 - 1;
      Vr[k2] = *(const u32x4_t*)(Vb + (size_t)row * HD);
    }
  };

  float m = -INFINITY, l = 0.f;
  f32x4_t O[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i) { const f32x4_t z = {0.f, 0.f, 0.f, 0.f}; O[i][0] = z; O[i][1] = z; }
  char* my = vt[wave];

  int t = wave;
  if (t < ntiles) load_tile(t);
  for (; t < ntiles; t += kWaves) {
    const int cnt = t1 - (t0 + t * kTok);               // tokens of this tile that exist (>= 1)
    // the previous tile's reads of the LDS region are done: their results fed its MFMAs
#pragma unroll
    for (int k2 = 0; k2 < 8; ++k2) *(u32x4_t*)(my + (4 * k2 + g) * kPitch + n * 16) = Vr[k2];
    f32x4_t sp[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
      sp[tt] = z;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        sp[tt] = Mfma<Tag>::run(A[ks][tt], qh[ks], sp[tt]);
        if (SPLIT) sp[tt] = Mfma<Tag>::run(A[ks][tt], ql[ks], sp[tt]);
      }
    }
    if (t + kWaves < ntiles) load_tile(t + kWaves);     // lands while this tile is finished
    // ---- softmax of head n: this lane holds tokens 4g+e (sp[0]) and 16+4g+e (sp[1])
    float s[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s[e] = 4 * g + e < cnt ? sp[0][e] : -INFINITY;
      s[4 + e] = 16 + 4 * g + e < cnt ? sp[1][e] : -INFINITY;
    }
    float tmax = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));            // finite: token 0 of the tile exists
    if (tmax > m) {                                      // same decision in the four lanes of a head
      const float alpha = fast_exp2(m - tmax);           // 0 on the first tile (m = -inf)
      m = tmax;
      l *= alpha;
#pragma unroll
      for (int i = 0; i < 4; ++i) { O[i][0] *= alpha; O[i][1] *= alpha; }
    }
    u32x4_t Phi, Plo = {0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float p0 = fast_exp2(s[2 * c] - m), p1 = fast_exp2(s[2 * c + 1] - m);
      Phi[c] = cvt_pack(p0, p1, Tag{});
      float k0 = lo_to_f32(Phi[c], Tag{}), k1 = hi_to_f32(Phi[c], Tag{});
      if (SPLIT) {
        Plo[c] = cvt_pack(p0 - k0, p1 - k1, Tag{});
        k0 += lo_to_f32(Plo[c], Tag{});
        k1 += hi_to_f32(Plo[c], Tag{});
      }
      l += k0 + k1;                                      // the sum uses the values the MFMA will see
    }
    // ---- O^T += V^T . P^T, 32 columns (16 dwords) at a time
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the tile is in LDS for every lane of the wave
    const char* vA = my + (4 * g) * kPitch + n * 4;
    const char* vB = vA + 16 * kPitch;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
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
      O[i][0] = Mfma<Tag>::run(te, Phi, O[i][0]);
      O[i][1] = Mfma<Tag>::run(to, Phi, O[i][1]);
      if (SPLIT) {
        O[i][0] = Mfma<Tag>::run(te, Plo, O[i][0]);
        O[i][1] = Mfma<Tag>::run(to, Plo, O[i][1]);
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next tile is written
  }

  // ---- this wave's part: O[i][j][e] is (head h0 + n, column 32 i + 8 g + 2 e + j)
  float lt = l + __shfl_xor(l, 16);
  lt += __shfl_xor(lt, 32);
  if (n < QG) {
    const size_t po = ((size_t)(su * kWaves + wave) * B + b) * H + h0 + n;
    const float inv = lt > 0.f ? 1.0f / lt : 0.f;        // a wave without tiles writes zeros and -inf
    float* orow = out_part + po * 128 + 8 * g;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f32x4_t v0 = {O[i][0][0] * inv, O[i][1][0] * inv, O[i][0][1] * inv, O[i][1][1] * inv};
      const f32x4_t v1 = {O[i][0][2] * inv, O[i][1][2] * inv, O[i][0][3] * inv, O[i][1][3] * inv};
      *(f32x4_t*)(orow + 32 * i) = v0;
      *(f32x4_t*)(orow + 32 * i + 4) = v1;
    }
    if (g == 0) lse_part[po] = lt > 0.f ? (m + log2f(lt)) * kLn2 : -INFINITY;
  }
}

}  // namespace

bool keyonly_mfma_applies(int H, int H_kv, int d, int r) { return d == 128 && r <= 128 && H / H_kv <= 16; }

// Splits of the token axis: about two workgroups per CU, at least two tiles per wave, at most
// 16 (four parts per split go to merge_parts, which takes 64).
int keyonly_mfma_splits(int B, int H_kv, int T) {
  const int wgs = B * H_kv;
  int s = (512 + wgs - 1) / wgs;
  const int by_len = T / (2 * kWaves * kTok);
  if (s > by_len) s = by_len;
  if (s > 16) s = 16;
  return s < 1 ? 1 : s;
}

ap_status launch_keyonly_mfma(ap_dtype dt, const uint16_t* Qp, const void* Ck, const void* V, float* out_part,
                              float* lse_part, int B, int H, int H_kv, int T, int T_cap, int r, int S,
                              hipStream_t stream) {
  const int QG = H / H_kv;
  const int per = ((T + S - 1) / S + kTok - 1) / kTok * kTok;
  const dim3 grid(8 * H_kv * ((B * S + 7) / 8));
  const int nks = (r + 31) / 32;
#define AP_KM(TAG, N)                                                                                       \
  hipLaunchKernelGGL((keyonly_mfma<TAG, N>), grid, dim3(256), 0, stream, Qp, (const uint16_t*)Ck,           \
                     (const uint16_t*)V, out_part, lse_part, B, H, QG, T, T_cap, r, S, per)
  if (dt == AP_F16) {
    switch (nks) { case 1: AP_KM(F16Tag, 1); break; case 2: AP_KM(F16Tag, 2); break; case 3: AP_KM(F16Tag, 3); break;
                   default: AP_KM(F16Tag, 4); break; }
  } else {
    switch (nks) { case 1: AP_KM(BF16Tag, 1); break; case 2: AP_KM(BF16Tag, 2); break; case 3: AP_KM(BF16Tag, 3); break;
                   default: AP_KM(BF16Tag, 4); break; }
  }
#undef AP_KM
  return AP_OK;
}

}  // namespace ap
