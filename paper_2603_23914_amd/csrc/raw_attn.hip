// The uncompressed segment of the cache (paper Alg. 1: C_u = {K, V}, the text tokens and the
// tokens generated since the last compression) and the merge of segments under one softmax.
//
//   raw_attn_partial   flash-decode over raw K, V [B, T_u_cap, HD] in 16-bit storage: a
//                      workgroup owns one head of one sequence and a range of tokens; groups
//                      of d/8 lanes take one token each (one 16-byte chunk of the head's key
//                      and value slice per lane), several tokens in flight per group, online
//                      softmax per group, groups combined through LDS at the end.
//   keyonly_partial    the same flash-decode for a cache whose KEYS are compressed (coefficients
//                      C_k [B, T_cap, r] and a basis) while its values stay raw (Sec. 4, the
//                      text-domain experiment compresses keys only, R_k = 64): the basis is
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

// grid (H, S, B), 256 threads.  LPH = d / 8 lanes form a group; G = 256 / LPH groups.  QG query
// heads share one key/value head (grouped queries; 1 = every head has its own).
// Split su covers tokens [su * per, min(T, (su + 1) * per)); group g takes every G-th of them.
// Writes the normalised partial output [su][b][h][d] and its log-sum-exp [su][b][h].
template <class Tag, int LPH>
__global__ void __launch_bounds__(256)
raw_attn_partial(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K,
                 const uint16_t* __restrict__ V, float* __restrict__ out_part,
                 float* __restrict__ lse_part, int B, int H, int QG, int T, int T_cap, int per,
                 float scale_log2) {
  constexpr int d = LPH * 8;
  constexpr int G = 256 / LPH;
  __shared__ float red[G][d + 2];
  const int h = blockIdx.x, su = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, g = tid / LPH, li = tid % LPH;
  const size_t HD = (size_t)(H / QG) * d;         // QG query heads share a key/value head
  const u32x4_t qv = *(const u32x4_t*)(q + ((size_t)b * H + h) * d + li * 8);
  const uint16_t* Kb = K + (size_t)b * T_cap * HD + (size_t)(h / QG) * d + li * 8;
  const uint16_t* Vb = V + (size_t)b * T_cap * HD + (size_t)(h / QG) * d + li * 8;
  const int t0 = su * per;
  int t1 = t0 + per;
  t1 = t1 < T ? t1 : T;

  float m = -INFINITY, l = 0.f;
  float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
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
      kv[u] = *(const u32x4_t*)(Kb + (size_t)tc * HD);
      vv[u] = *(const u32x4_t*)(Vb + (size_t)tc * HD);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      float s = group_sum<LPH>(dot8<Tag>(kv[u], qv, 0.f)) * scale_log2;
      if (tok[u] >= t1) s = -INFINITY;                 // same decision in all lanes of the group
      const float m_new = fmaxf(m, s);
      if (m_new > -INFINITY) {
        const float alpha = fast_exp2(m - m_new);
        const float pw = fast_exp2(s - m_new);
        l = l * alpha + pw;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[2 * e] = o[2 * e] * alpha + pw * lo_to_f32(vv[u][e], Tag{});
          o[2 * e + 1] = o[2 * e + 1] * alpha + pw * hi_to_f32(vv[u][e], Tag{});
        }
        m = m_new;
      }
    }
  }
  // ---- combine the groups
#pragma unroll
  for (int e = 0; e < 8; ++e) red[g][li * 8 + e] = o[e];
  if (li == 0) { red[g][d] = m; red[g][d + 1] = l; }
  __syncthreads();
  float mstar = -INFINITY;
  for (int k = 0; k < G; ++k) mstar = fmaxf(mstar, red[k][d]);
  const size_t po = ((size_t)su * B + b) * H + h;
  if (mstar == -INFINITY) {                              // no token in this range
    if (tid < d) out_part[po * d + tid] = 0.f;
    if (tid == 0) lse_part[po] = -INFINITY;
    return;
  }
  if (tid < d) {
    float acc = 0.f, L = 0.f;
    for (int k = 0; k < G; ++k) {
      const float w = fast_exp2(red[k][d] - mstar);       // 0 for a group without tokens
      acc = fmaf(w, red[k][tid], acc);
      L = fmaf(w, red[k][d + 1], L);
    }
    out_part[po * d + tid] = acc / L;
    if (tid == 0) lse_part[po] = (mstar + log2f(L)) * kLn2;
  }
}

// Key-only compression.  grid (S, H, B), 256 threads; the split index varies fastest, and S is a
// multiple of 8 whenever there is more than one split, so the workgroups of all heads that
// walk one token range sit on the same XCD and find its coefficient rows (shared by every
// head) and value slices (shared by the heads of a group) in that XCD's L2.
// Qp [B][2][H][r]: the folded queries as hi + lo 16-bit pairs, softmax scale and log2(e)
// included.  A group of LPH lanes takes a token: lane li holds the value chunk li and the
// coefficient chunks li, li + LPH, ... (16 bytes each; NCH of them, those at or beyond r / 8
// re-read chunk 0 against a zero query).  KU tokens are in flight per group.
template <class Tag, int LPH, int NCH, int KU>
__global__ void __launch_bounds__(256)
keyonly_partial(const uint16_t* __restrict__ Qp, const uint16_t* __restrict__ Ck,
                const uint16_t* __restrict__ V, float* __restrict__ out_part,
                float* __restrict__ lse_part, int B, int H, int QG, int T, int T_cap, int r, int per) {
  constexpr int d = LPH * 8;
  constexpr int G = 256 / LPH;
  __shared__ float red[G][d + 2];
  const int su = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, g = tid / LPH, li = tid % LPH;
  const size_t HD = (size_t)(H / QG) * d;
  const int nchunk = r >> 3;
  u32x4_t qh[NCH], ql[NCH];
  uint32_t coff[NCH];                               // element offset of the lane's chunks in a row
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int k = li + LPH * c;
    const u32x4_t z = {0, 0, 0, 0};
    qh[c] = z; ql[c] = z; coff[c] = 0;
    if (k < nchunk) {
      const uint16_t* qp = Qp + (((size_t)b * 2) * H + h) * r + k * 8;
      qh[c] = *(const u32x4_t*)qp;
      ql[c] = *(const u32x4_t*)(qp + (size_t)H * r);
      coff[c] = (uint32_t)k * 8u;
    }
  }
  const uint16_t* Cb = Ck + (size_t)b * T_cap * r;
  const uint16_t* Vb = V + (size_t)b * T_cap * HD + (size_t)(h / QG) * d + li * 8;
  const int t0 = su * per;
  int t1 = t0 + per;
  t1 = t1 < T ? t1 : T;

  float m = -INFINITY, l = 0.f;
  float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const int ntok = t1 - t0;
  const int rounds = ntok > 0 ? (ntok + G * KU - 1) / (G * KU) : 0;
  for (int rd = 0; rd < rounds; ++rd) {
    u32x4_t cv[KU][NCH], vv[KU];
    int tok[KU];
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      tok[u] = t0 + (rd * KU + u) * G + g;
      const int tc = tok[u] < t1 ? tok[u] : t1 - 1;      // in-bounds repeat, masked below
      const uint16_t* crow = Cb + (size_t)tc * r;
#pragma unroll
      for (int c = 0; c < NCH; ++c) cv[u][c] = *(const u32x4_t*)(crow + coff[c]);
      vv[u] = *(const u32x4_t*)(Vb + (size_t)tc * HD);
    }
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      float part = 0.f;
#pragma unroll
      for (int c = 0; c < NCH; ++c) part = dot8<Tag>(cv[u][c], ql[c], dot8<Tag>(cv[u][c], qh[c], part));
      float s = group_sum<LPH>(part);
      if (tok[u] >= t1) s = -INFINITY;                   // same decision in all lanes of the group
      const float m_new = fmaxf(m, s);
      if (m_new > -INFINITY) {
        const float alpha = fast_exp2(m - m_new);
        const float pw = fast_exp2(s - m_new);
        l = l * alpha + pw;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[2 * e] = o[2 * e] * alpha + pw * lo_to_f32(vv[u][e], Tag{});
          o[2 * e + 1] = o[2 * e + 1] * alpha + pw * hi_to_f32(vv[u][e], Tag{});
        }
        m = m_new;
      }
    }
  }
  // ---- combine the groups (as raw_attn_partial)
#pragma unroll
  for (int e = 0; e < 8; ++e) red[g][li * 8 + e] = o[e];
  if (li == 0) { red[g][d] = m; red[g][d + 1] = l; }
  __syncthreads();
  float mstar = -INFINITY;
  for (int k = 0; k < G; ++k) mstar = fmaxf(mstar, red[k][d]);
  const size_t po = ((size_t)su * B + b) * H + h;
  if (mstar == -INFINITY) {                              // no token in this range
    if (tid < d) out_part[po * d + tid] = 0.f;
    if (tid == 0) lse_part[po] = -INFINITY;
    return;
  }
  if (tid < d) {
    float acc = 0.f, L = 0.f;
    for (int k = 0; k < G; ++k) {
      const float w = fast_exp2(red[k][d] - mstar);
      acc = fmaf(w, red[k][tid], acc);
      L = fmaf(w, red[k][d + 1], L);
    }
    out_part[po * d + tid] = acc / L;
    if (tid == 0) lse_part[po] = (mstar + log2f(L)) * kLn2;
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

// grid (ceil(H d / 256), B), 256 threads: one output element per thread.
template <class Tag, bool OUT_F32>
__global__ void __launch_bounds__(256)
merge_parts(const MergeArgs a, void* __restrict__ out, float* __restrict__ lse, int H, int d) {
  const int b = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
  if (i >= H * d) return;
  const int h = i / d;
  const size_t lo = (size_t)b * H + h, oo = (size_t)b * H * d + i;
  float m = -INFINITY;
  for (int k = 0; k < kMaxLists; ++k)
    for (int c = 0; c < a.cnt[k]; ++c) m = fmaxf(m, a.lse[k][lo + c * a.lstride]);
  float acc = 0.f, z = 0.f;
  if (m > -INFINITY) {
    for (int k = 0; k < kMaxLists; ++k)
      for (int c = 0; c < a.cnt[k]; ++c) {
        const float w = __expf(a.lse[k][lo + c * a.lstride] - m);
        acc = fmaf(w, a.out[k][oo + c * a.ostride], acc);
        z += w;
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

int raw_splits(int B, int H, int d, int T) {
  // about four workgroups per CU; a split holds at least one round of every group
  const int G = 256 / (d / 8);
  int s = (1024 + B * H - 1) / (B * H);
  const int by_len = (T + G * kUnroll - 1) / (G * kUnroll);
  if (s > by_len) s = by_len;
  if (s > 64) s = 64;
  return s < 1 ? 1 : s;
}

template <class Tag>
void launch_raw_partial(const void* q, const void* K, const void* V, float* op, float* lp, int B, int H,
                        int G, int d, int T, int T_cap, int S, float sm_scale, hipStream_t stream) {
  const int per = (T + S - 1) / S;
  const dim3 grid(H, S, B);
  const float sc = sm_scale * kLog2e;
#define AP_RAW(L)                                                                               \
  hipLaunchKernelGGL((raw_attn_partial<Tag, L>), grid, dim3(256), 0, stream, (const uint16_t*)q, \
                     (const uint16_t*)K, (const uint16_t*)V, op, lp, B, H, G, T, T_cap, per, sc)
  switch (d) {
    case 32: AP_RAW(4); break;
    case 64: AP_RAW(8); break;
    case 128: AP_RAW(16); break;
    default: AP_RAW(32); break;
  }
#undef AP_RAW
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
int keyonly_splits(int B, int H, int d, int T) {
  const int G = 256 / (d / 8);
  int s = (1024 + B * H - 1) / (B * H);
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
  const dim3 grid(S, H, B);
  const int nch = ((r >> 3) + LPH - 1) / LPH;          // 16-byte coefficient chunks per lane
#define AP_KO(N, U)                                                                                  \
  if (nch <= N) {                                                                                    \
    hipLaunchKernelGGL((keyonly_partial<Tag, LPH, N, U>), grid, dim3(256), 0, stream, Qp,            \
                       (const uint16_t*)Ck, (const uint16_t*)V, op, lp, B, H, QG, T, T_cap, r, per); \
    return AP_OK;                                                                                    \
  }
  AP_KO(1, 4) AP_KO(2, 4) AP_KO(3, 2)
  if constexpr (LPH <= 16) { AP_KO(5, 2) }
  if constexpr (LPH <= 8) { AP_KO(10, 1) }
  if constexpr (LPH <= 4) { AP_KO(20, 1) }
#undef AP_KO
  set_error("ap_keyonly_attn: r=%d too large for d=%d", r, LPH * 8);
  return AP_ERR_UNSUPPORTED;
}

}  // namespace

size_t raw_attn_workspace(int B, int H, int d, int T) {
  const int S = raw_splits(B, H, d, T);
  return round_up((size_t)S * B * H * d * 4, 256) + round_up((size_t)S * B * H * 4, 256);
}

ap_status launch_raw_attn(const void* q, const void* K, const void* V, float* out, float* lse, int B,
                          int H, int H_kv, int d, int T, int T_cap, float sm_scale, ap_dtype dt,
                          void* workspace, hipStream_t stream) {
  const int G = H / H_kv;
  const int S = raw_splits(B, H, d, T);
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

size_t keyonly_attn_workspace(int B, int H, int d, int T, int r) {
  const int S = keyonly_splits(B, H, d, T);
  return keyonly_qp_bytes(B, H, r) + round_up((size_t)S * B * H * d * 4, 256) +
         round_up((size_t)S * B * H * 4, 256);
}

ap_status launch_keyonly_attn(const void* q, const void* Ck, const void* Bk, int64_t bstride, const void* V,
                              float* out, float* lse, int B, int H, int H_kv, int d, int T, int T_cap, int r,
                              float sm_scale, ap_dtype dt, void* workspace, hipStream_t stream) {
  const int QG = H / H_kv;
  const int S = keyonly_splits(B, H, d, T);
  char* ws = (char*)workspace;
  uint16_t* Qp = (uint16_t*)ws;
  float* parts = (float*)(ws + keyonly_qp_bytes(B, H, r));
  float* lparts = (float*)(ws + keyonly_qp_bytes(B, H, r) + round_up((size_t)S * B * H * d * 4, 256));
  // q' = scale * log2(e) * B_k[:, slice] q_h for every head, written as hi + lo pairs
  ap_status st = launch_fold_heads(dt, Bk, bstride, q, Qp, B, H, H_kv, H, d, r, sm_scale * kLog2e, stream);
  if (st != AP_OK) return st;
  float* op = S > 1 ? parts : out;
  float* lp = (S > 1 || !lse) ? lparts : lse;
#define AP_KL(TAG)                                                                                          \
  switch (d) {                                                                                              \
    case 32: st = launch_keyonly_partial<TAG, 4>(Qp, Ck, V, op, lp, B, H, QG, T, T_cap, r, S, stream); break;  \
    case 64: st = launch_keyonly_partial<TAG, 8>(Qp, Ck, V, op, lp, B, H, QG, T, T_cap, r, S, stream); break;  \
    case 128: st = launch_keyonly_partial<TAG, 16>(Qp, Ck, V, op, lp, B, H, QG, T, T_cap, r, S, stream); break; \
    default: st = launch_keyonly_partial<TAG, 32>(Qp, Ck, V, op, lp, B, H, QG, T, T_cap, r, S, stream); break; \
  }
  if (dt == AP_F16) { AP_KL(F16Tag) } else { AP_KL(BF16Tag) }
#undef AP_KL
  if (st != AP_OK) return st;
  if (S > 1) {
    MergeArgs a{{op, nullptr}, {lp, nullptr}, {S, 0}, (size_t)B * H * d, (size_t)B * H};
    launch_merge<F16Tag>(a, out, true, lse, B, H, d, stream);
  }
  return check_launch("ap_keyonly_attn");
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
