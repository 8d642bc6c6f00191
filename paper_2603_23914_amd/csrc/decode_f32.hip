// Decode attention over fp32 coefficients and bases: simple kernels for small
// cases (the fp32 parity configuration), any shape, per-token ranks read directly.
//
// Same algebra as the fast path (paper Alg. 1 with the decompression matrices
// absorbed by associativity):
//   q'[h,j]  = sm_scale * sum_i Bk[j, h*d+i] q[h,i]
//   s[h,t]   = sum_{j<rk_t} Ck[t,j] q'[h,j]
//   p[h,:]   = softmax_t s[h,:]
//   u[h,j]   = sum_{t: rv_t>j} p[h,t] Cv[t,j]
//   out[h,i] = sum_j u[h,j] Bv[j, h*d+i]
// Long sums are carried in fp64 so that results are independent of T.
#include "ap_common.hpp"

namespace ap {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ double block_reduce_sum(double v, double* sh) {
  const int tid = threadIdx.x;
  sh[tid] = v;
  __syncthreads();
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if (tid < s) sh[tid] += sh[tid + s];
    __syncthreads();
  }
  double r = sh[0];
  __syncthreads();
  return r;
}
__device__ __forceinline__ float block_reduce_max(float v, float* sh) {
  const int tid = threadIdx.x;
  sh[tid] = v;
  __syncthreads();
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if (tid < s) sh[tid] = fmaxf(sh[tid], sh[tid + s]);
    __syncthreads();
  }
  float r = sh[0];
  __syncthreads();
  return r;
}

// grid (H, B): q' for one head.
__global__ void __launch_bounds__(kThreads)
f32_fold(const float* __restrict__ q, const float* __restrict__ Bk, int64_t bstride,
         float* __restrict__ qp, int H, int G, int d, int r, float sm_scale) {
  const int h = blockIdx.x, b = blockIdx.y;
  const float* qh = q + ((size_t)b * H + h) * d;
  const float* Bb = Bk + (size_t)b * bstride;
  const size_t HD = (size_t)(H / G) * d;          // G query heads share a key/value head
  for (int j = threadIdx.x; j < r; j += kThreads) {
    const float* row = Bb + (size_t)j * HD + (size_t)(h / G) * d;
    double acc = 0.0;
    for (int i = 0; i < d; ++i) acc += (double)row[i] * (double)qh[i];
    qp[((size_t)b * H + h) * r + j] = (float)(acc * (double)sm_scale);
  }
}

// grid (ceil(T/kThreads), H, B): scores.
__global__ void __launch_bounds__(kThreads)
f32_scores(const float* __restrict__ Ck, const float* __restrict__ qp,
           const int32_t* __restrict__ rank_k, float* __restrict__ S,
           float* __restrict__ scores, int H, int T, int T_cap, int r) {
  const int t = blockIdx.x * kThreads + threadIdx.x;
  const int h = blockIdx.y, b = blockIdx.z;
  if (t >= T) return;
  const float* row = Ck + ((size_t)b * T_cap + t) * r;
  const float* qh = qp + ((size_t)b * H + h) * r;
  int rk = rank_k ? rank_k[(size_t)b * T + t] : r;
  rk = rk < 0 ? 0 : (rk > r ? r : rk);
  double acc = 0.0;
  for (int j = 0; j < rk; ++j) acc += (double)row[j] * (double)qh[j];
  S[((size_t)b * H + h) * T + t] = (float)acc;
  if (scores) scores[((size_t)b * T_cap + t) * H + h] = (float)acc;     // [B][T_cap][H]
}

// grid (H, B): softmax, weighted coefficient sum, expansion through Bv.
__global__ void __launch_bounds__(kThreads)
f32_softmax_out(const float* __restrict__ Cv, const float* __restrict__ Bv, int64_t bstride,
                const int32_t* __restrict__ rank_v, float* __restrict__ S,
                float* __restrict__ U, float* __restrict__ out, float* __restrict__ lse, int H,
                int G, int d, int T, int T_cap, int r) {
  __shared__ double shd[kThreads];
  __shared__ float shf[kThreads];
  const int h = blockIdx.x, b = blockIdx.y;
  float* s = S + ((size_t)b * H + h) * T;
  float m = -INFINITY;
  for (int t = threadIdx.x; t < T; t += kThreads) m = fmaxf(m, s[t]);
  m = block_reduce_max(m, shf);
  double z = 0.0;
  for (int t = threadIdx.x; t < T; t += kThreads) {
    float e = expf(s[t] - m);
    s[t] = e;
    z += (double)e;
  }
  z = block_reduce_sum(z, shd);  // also orders the writes to s[] before the reads below
  if (threadIdx.x == 0 && lse) lse[(size_t)b * H + h] = m + (float)log(z);
  const double inv = 1.0 / z;
  float* u = U + ((size_t)b * H + h) * r;
  const float* Cb = Cv + (size_t)b * T_cap * r;
  for (int j = threadIdx.x; j < r; j += kThreads) {
    double acc = 0.0;
    for (int t = 0; t < T; ++t) {
      int rv = rank_v ? rank_v[(size_t)b * T + t] : r;
      if (j < rv) acc += (double)s[t] * (double)Cb[(size_t)t * r + j];
    }
    u[j] = (float)(acc * inv);
  }
  __syncthreads();
  const float* Bb = Bv + (size_t)b * bstride;
  const size_t HD = (size_t)(H / G) * d;
  for (int i = threadIdx.x; i < d; i += kThreads) {
    double acc = 0.0;
    for (int j = 0; j < r; ++j) acc += (double)u[j] * (double)Bb[(size_t)j * HD + (size_t)(h / G) * d + i];
    out[((size_t)b * H + h) * d + i] = (float)acc;
  }
}

}  // namespace

size_t decode_f32_workspace(int B, int H, int d, int T, int r) {
  (void)d;
  size_t qp = round_up((size_t)B * H * r * 4, 256);
  size_t S = round_up((size_t)B * H * T * 4, 256);
  size_t U = round_up((size_t)B * H * r * 4, 256);
  return qp + S + U;
}

ap_status launch_decode_f32(const DecodeArgs& a) {
  AP_REQUIRE(a.dt_coef == AP_F32, AP_ERR_INVALID_ARG, "ap_decode_attn: fp32 path needs fp32 coefficients");
  AP_REQUIRE(a.H <= 65535 && a.B <= 65535, AP_ERR_UNSUPPORTED, "ap_decode_attn: H, B must be <= 65535");
  char* ws = (char*)a.workspace;
  float* qp = (float*)ws;
  ws += round_up((size_t)a.B * a.H * a.r * 4, 256);
  float* S = (float*)ws;
  ws += round_up((size_t)a.B * a.H * a.T * 4, 256);
  float* U = (float*)ws;
  hipLaunchKernelGGL(f32_fold, dim3(a.H, a.B), dim3(kThreads), 0, a.stream, (const float*)a.q,
                     (const float*)a.Bk, a.basis_batch_stride, qp, a.H, a.H / a.H_kv, a.d, a.r, a.sm_scale);
  hipLaunchKernelGGL(f32_scores, dim3((a.T + kThreads - 1) / kThreads, a.H, a.B), dim3(kThreads), 0,
                     a.stream, (const float*)a.Ck, qp, a.rank_k, S, a.scores, a.H, a.T, a.T_cap, a.r);
  hipLaunchKernelGGL(f32_softmax_out, dim3(a.H, a.B), dim3(kThreads), 0, a.stream,
                     (const float*)a.Cv, (const float*)a.Bv, a.basis_batch_stride, a.rank_v, S, U,
                     (float*)a.out, a.lse, a.H, a.H / a.H_kv, a.d, a.T, a.T_cap, a.r);
  return check_launch("ap_decode_attn(fp32)");
}

}  // namespace ap
