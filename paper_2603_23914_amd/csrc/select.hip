// Attention-aware rank groups (paper Sec. 3.2; Alg. 1 "determine the tokens m_f for each
// group f based on I").
//
// Per batch row the tokens are ordered by (importance descending, token index ascending)
// and cut at fixed sorted positions into F groups.  Nothing is sorted: a group boundary at
// sorted position p is fully described by the p-th largest key kappa and by how many of the
// tokens whose key equals kappa still fall in front of it (the quota), so
//   1. an 8-bit-digit radix select finds (kappa, quota) of all F-1 boundaries at once
//      (four passes over the row, histograms in LDS);
//   2. every thread owns a contiguous run of tokens; block-wide prefix sums of "key == kappa"
//      give each token its position among equal keys, which decides its group;
//   3. block-wide prefix sums of the group counts give each token its slot in its group's
//      ascending index list.
// One workgroup of 1024 threads per batch row; rows of up to 32768 tokens are first copied to
// LDS as sort keys, so the four radix passes and the two walks read LDS, not memory.  All
// integer work, results are unique.
#include "ap_common.hpp"

namespace ap {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxF = 8;
constexpr uint32_t kNone = 0xffffffffu;

struct SelectParams {
  const float* mass;
  int T, F;
  int32_t bound[kMaxF + 1];   // sorted-position cuts: bound[0] = 0, bound[F] = T
  int32_t grank[kMaxF];
  int32_t* rank_out;
  int32_t* bucket_off;
  int32_t* bucket_idx;
};

// Order-preserving map float -> uint32 (larger value, larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t key_of(float m) {
  uint32_t u = __builtin_bit_cast(uint32_t, m);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Histogram increment with same-digit lanes of a wave combined (importance values share
// their leading bits, so the first passes would otherwise serialise on a few counters).
// Every lane of the wave must call this; d == kNone means "nothing to count".
__device__ __forceinline__ void hist_add(uint32_t* h, uint32_t d) {
  const int lane = threadIdx.x & 63;
#pragma unroll 1
  for (int it = 0; it < 4; ++it) {
    const unsigned long long act = __ballot(d != kNone);
    if (act == 0ull) return;
    const int leader = __ffsll((long long)act) - 1;
    const uint32_t dl = (uint32_t)__shfl((int)d, leader);
    const unsigned long long same = __ballot(d == dl);
    if (lane == leader) atomicAdd(&h[dl], (uint32_t)__popcll(same));
    if (d == dl) d = kNone;
  }
  if (d != kNone) atomicAdd(&h[d], 1u);
}

// Exclusive prefix sum of one int per thread over the workgroup (thread order); *total
// receives the workgroup sum.  wave_tot: kWaves ints of LDS.  Two barriers.
__device__ __forceinline__ int block_excl_scan(int v, int* wave_tot, int* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();                       // previous use of wave_tot is over
  if (lane == 63) wave_tot[w] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) {
    const int x = wave_tot[i];
    if (i < w) base += x;
    tot += x;
  }
  *total = tot;
  return base + incl - v;
}

constexpr int kStagedMax = 32768;      // tokens whose keys fit the dynamic LDS slice (128 KiB)

template <bool STAGED>
__global__ void __launch_bounds__(kThreads) select_ranks_kernel(const SelectParams p) {
  extern __shared__ __attribute__((aligned(16))) uint32_t keys_lds[];   // STAGED: [T]
  __shared__ uint32_t hist[kMaxF - 1][256];
  __shared__ uint32_t s_prefix[kMaxF - 1];   // key bits fixed so far (kappa after pass 4)
  __shared__ uint32_t s_need[kMaxF - 1];     // 1-based position still to find (quota after pass 4)
  __shared__ int wave_tot[kWaves];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int b = blockIdx.x, T = p.T, F = p.F, nb = F - 1;
  const float* m = p.mass + (size_t)b * T;
  if (STAGED) {
    for (int t = tid; t < T; t += kThreads) keys_lds[t] = key_of(m[t]);
    __syncthreads();
  }
  auto key_at = [&](int t) -> uint32_t { return STAGED ? keys_lds[t] : key_of(m[t]); };

  // a cut at 0 or at T needs no threshold search
  bool active[kMaxF - 1];
#pragma unroll
  for (int g = 0; g < kMaxF - 1; ++g) active[g] = g < nb && p.bound[g + 1] > 0 && p.bound[g + 1] < T;
  if (tid < kMaxF - 1) {
    uint32_t need = 0u;
#pragma unroll
    for (int g = 0; g < kMaxF - 1; ++g) need = (tid == g && g < nb) ? (uint32_t)p.bound[g + 1] : need;
    s_prefix[tid] = 0u;
    s_need[tid] = need;
  }

  // ---- 1. radix select, most significant digit first
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int i = tid; i < (kMaxF - 1) * 256; i += kThreads) (&hist[0][0])[i] = 0u;
    __syncthreads();
    uint32_t pre[kMaxF - 1];
#pragma unroll
    for (int g = 0; g < kMaxF - 1; ++g) pre[g] = s_prefix[g];
    const int Tpad = (T + 63) & ~63;     // whole waves stay in the loop (hist_add uses ballots)
    for (int t = tid; t < Tpad; t += kThreads) {
      const bool in = t < T;
      const uint32_t key = in ? key_at(t) : 0u;
      const uint32_t dig = (key >> shift) & 255u;
      if (pass == 0) {
        hist_add(hist[0], in ? dig : kNone);       // every boundary shares the empty prefix
      } else {
        // few keys still match a boundary's prefix: plain atomics
        const uint32_t hi = key >> (shift + 8);
#pragma unroll
        for (int g = 0; g < kMaxF - 1; ++g) {
          if (active[g] && in && hi == (pre[g] >> (shift + 8))) atomicAdd(&hist[g][dig], 1u);
        }
      }
    }
    __syncthreads();
    // wave g walks boundary g's histogram from the top: lane l owns digits 4l .. 4l+3
    bool act_w = false;
#pragma unroll
    for (int g = 0; g < kMaxF - 1; ++g) act_w = act_w || (w == g && active[g]);
    if (act_w) {
      const uint32_t* h = hist[pass == 0 ? 0 : w];
      uint32_t c[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) c[j] = h[4 * lane + j];
      const uint32_t tot = c[0] + c[1] + c[2] + c[3];
      uint32_t incl = tot;               // sum over lanes >= lane
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t dn = (uint32_t)__shfl_down((int)incl, o);
        if (lane + o < 64) incl += dn;
      }
      const uint32_t above = incl - tot;
      const uint32_t k = s_need[w];
      if (above < k && k <= incl) {      // exactly one lane
        uint32_t acc = above, digit = 0, left = k;
        bool found = false;
#pragma unroll
        for (int j = 3; j >= 0; --j) {
          if (!found) {
            if (k <= acc + c[j]) { digit = 4 * lane + j; left = k - acc; found = true; }
            else acc += c[j];
          }
        }
        s_prefix[w] = s_prefix[w] | (digit << shift);
        s_need[w] = left;
      }
    }
    __syncthreads();
  }

  uint32_t kappa[kMaxF - 1], quota[kMaxF - 1];
#pragma unroll
  for (int g = 0; g < kMaxF - 1; ++g) {
    kappa[g] = kNone; quota[g] = 0u;                       // cut at 0 (or unused): nobody in front
    if (g < nb) {
      if (active[g]) { kappa[g] = s_prefix[g]; quota[g] = s_need[g]; }
      else if (p.bound[g + 1] >= T) { kappa[g] = 0u; quota[g] = (uint32_t)T; }   // cut at T: everybody
    }
  }

  // ---- 2. position among equal keys -> group of every token
  const int chunk = (T + kThreads - 1) / kThreads;
  const int t0 = min(T, tid * chunk), t1 = min(T, t0 + chunk);
  int eq[kMaxF - 1];
#pragma unroll
  for (int g = 0; g < kMaxF - 1; ++g) eq[g] = 0;
  for (int t = t0; t < t1; ++t) {
    const uint32_t key = key_at(t);
#pragma unroll
    for (int g = 0; g < kMaxF - 1; ++g) eq[g] += (key == kappa[g]) ? 1 : 0;
  }
  int dummy;
#pragma unroll
  for (int g = 0; g < kMaxF - 1; ++g)
    if (g < nb) eq[g] = block_excl_scan(eq[g], wave_tot, &dummy);   // now: equal keys before t0
  int cnt[kMaxF];
#pragma unroll
  for (int g = 0; g < kMaxF; ++g) cnt[g] = 0;
  int32_t* rank_row = p.rank_out + (size_t)b * T;
  for (int t = t0; t < t1; ++t) {
    const uint32_t key = key_at(t);
    int grp = nb;
#pragma unroll
    for (int g = kMaxF - 2; g >= 0; --g) {
      const bool same = key == kappa[g];
      const bool in_front = key > kappa[g] || (same && (uint32_t)eq[g] < quota[g]);
      if (g < nb && in_front) grp = g;                      // membership is nested: keep the smallest
      eq[g] += same ? 1 : 0;
    }
    rank_row[t] = grp;                                      // group id for now, rank below
#pragma unroll
    for (int g = 0; g < kMaxF; ++g) cnt[g] += (grp == g) ? 1 : 0;
  }

  // ---- 3. slot inside the group's ascending index list
#pragma unroll
  for (int g = 0; g < kMaxF; ++g)
    if (g < F) cnt[g] = block_excl_scan(cnt[g], wave_tot, &dummy);
  int32_t* idx_row = p.bucket_idx + (size_t)b * T;
  for (int t = t0; t < t1; ++t) {
    const int grp = rank_row[t];
    int slot = 0, rk = 0;
#pragma unroll
    for (int g = 0; g < kMaxF; ++g) {
      if (grp == g) { slot = p.bound[g] + cnt[g]; rk = p.grank[g]; cnt[g] += 1; }
    }
    rank_row[t] = rk;
    if (slot < T) idx_row[slot] = t;    // always true; keeps a logic error inside the buffer
  }
  int cut = 0;
#pragma unroll
  for (int g = 0; g <= kMaxF; ++g) cut = tid == g ? p.bound[g] : cut;
  if (tid <= F) p.bucket_off[(size_t)b * (F + 1) + tid] = cut;
}

// Importance update of Eq. 1 for one new query: the attention weights of the query, averaged
// over the heads, enter the moving average.  grid (ceil(T / 256), B), one thread per token.
__global__ void __launch_bounds__(256)
update_importance_kernel(const float* __restrict__ scores, const float* __restrict__ lse,
                         float* __restrict__ mass, int H, int T, int T_cap, int64_t mass_stride,
                         float alpha) {
  const int t = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
  if (t >= T) return;
  const float* s = scores + (size_t)b * H * T_cap + t;
  const float* l = lse + (size_t)b * H;
  float acc = 0.f;
  int h = 0;
  for (; h + 8 <= H; h += 8) {                 // 8 independent loads in flight per thread
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = s[(size_t)(h + i) * T_cap];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += __expf(v[i] - l[h + i]);
  }
  for (; h < H; ++h) acc += __expf(s[(size_t)h * T_cap] - l[h]);
  float* m = mass + (size_t)b * mass_stride + t;
  *m = alpha * *m + (1.0f - alpha) * (acc / (float)H);
}

}  // namespace

ap_status launch_update_importance(const float* scores, const float* lse, float* mass, int B, int H,
                                   int T, int T_cap, int64_t mass_stride, float alpha,
                                   hipStream_t stream) {
  hipLaunchKernelGGL(update_importance_kernel, dim3((T + 255) / 256, B), dim3(256), 0, stream, scores,
                     lse, mass, H, T, T_cap, mass_stride, alpha);
  return check_launch("ap_update_importance");
}

size_t select_workspace(int, int, int) { return 256; }   // every intermediate lives in LDS

ap_status launch_select_ranks(const float* mass, int B, int T, int F, const int32_t* group_rank,
                              const int32_t* cum_num, int32_t den, int32_t* rank_out,
                              int32_t* bucket_off, int32_t* bucket_idx, void* ws,
                              hipStream_t stream) {
  (void)ws;
  AP_REQUIRE(T <= (1 << 30), AP_ERR_UNSUPPORTED, "ap_select_ranks: T must be <= 2^30");
  SelectParams p;
  p.mass = mass;
  p.T = T;
  p.F = F;
  p.bound[0] = 0;
  for (int g = 0; g < kMaxF; ++g) {
    p.bound[g + 1] = g < F ? (int32_t)(((int64_t)T * cum_num[g]) / den) : T;
    p.grank[g] = g < F ? group_rank[g] : 0;
  }
  p.rank_out = rank_out;
  p.bucket_off = bucket_off;
  p.bucket_idx = bucket_idx;
  if (T <= kStagedMax) {
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute((const void*)select_ranks_kernel<true>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, kStagedMax * 4);
      if (e != hipSuccess) {
        set_error("hipFuncSetAttribute: %s", hipGetErrorString(e));
        return AP_ERR_HIP;
      }
      attr_set = true;
    }
    hipLaunchKernelGGL(select_ranks_kernel<true>, dim3(B), dim3(kThreads), (size_t)T * 4, stream, p);
  } else {
    hipLaunchKernelGGL(select_ranks_kernel<false>, dim3(B), dim3(kThreads), 0, stream, p);
  }
  return check_launch("ap_select_ranks");
}

}  // namespace ap
