// Attention-aware rank groups (paper Sec. 3.2; Alg. 1 "determine the tokens m_f for each
// group f based on I").
//
// Per batch row the tokens are ordered by (importance descending, token index ascending)
// and cut at fixed sorted positions into F groups.  Nothing is sorted: a group boundary at
// sorted position p is fully described by the p-th largest key kappa and by how many of the
// tokens whose key equals kappa still fall in front of it (the quota), so
//   1. a radix select finds (kappa, quota) of all F-1 boundaries at once (four passes over
//      the row with digits of 12, 8, 8 and 4 bits, histograms in LDS);
//   2. every thread owns a contiguous run of tokens; block-wide prefix sums of "key == kappa"
//      give each token its position among equal keys, which decides its group;
//   3. block-wide prefix sums of the group counts give each token its slot in its group's
//      ascending index list.
// One workgroup of 1024 threads per batch row; rows of up to 32768 tokens are first copied to
// LDS as sort keys, so the four radix passes and the two walks read LDS, not memory.  The LDS
// copy skips one word after every 32 tokens: a thread's contiguous run of tokens then starts
// in a different bank than its neighbours' and the walks are free of bank conflicts.  Group
// ids replace the keys in that copy once they are known, and the ranks leave in a coalesced
// pass.  All integer work, results are unique.
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

// The same for N values per thread at once (two barriers for all of them).  wave_tot: N * kWaves ints.
template <int N>
__device__ __forceinline__ void block_excl_scan_n(int (&v)[N], int* wave_tot) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl[N];
#pragma unroll
  for (int k = 0; k < N; ++k) incl[k] = v[k];
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const int up = __shfl_up(incl[k], o);
      if (lane >= o) incl[k] += up;
    }
  }
  __syncthreads();                       // previous use of wave_tot is over
  if (lane == 63) {
#pragma unroll
    for (int k = 0; k < N; ++k) wave_tot[k * kWaves + w] = incl[k];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < N; ++k) {
    int base = 0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) {
      const int x = wave_tot[k * kWaves + i];
      if (i < w) base += x;
    }
    v[k] = base + incl[k] - v[k];
  }
}

constexpr int kStagedMax = 32768;      // tokens whose keys fit the dynamic LDS slice (132 KiB with padding)

template <bool STAGED>
__global__ void __launch_bounds__(kThreads) select_ranks_kernel(const SelectParams p) {
  extern __shared__ __attribute__((aligned(16))) uint32_t keys_lds[];   // STAGED: [T]
  __shared__ uint32_t hist[kMaxF - 1][256];
  __shared__ uint32_t hist0[4096];           // first pass: 12-bit digits, shared by all boundaries
  __shared__ uint32_t mark[128];             // one bit per first digit: some boundary's prefix
  __shared__ uint32_t s_prefix[kMaxF - 1];   // key bits fixed so far (kappa after pass 4)
  __shared__ uint32_t s_need[kMaxF - 1];     // 1-based position still to find (quota after pass 4)
  __shared__ int wave_tot[kMaxF * kWaves];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int b = blockIdx.x, T = p.T, F = p.F, nb = F - 1;
  const float* m = p.mass + (size_t)b * T;
  auto slot_of = [](int t) -> int { return t + (t >> 5); };      // one pad word per 32 tokens
  if (STAGED) {
    for (int t0 = tid; t0 < T; t0 += 8 * kThreads) {        // eight loads in flight per thread
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int t = t0 + u * kThreads;
        v[u] = m[t < T ? t : T - 1];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int t = t0 + u * kThreads;
        if (t < T) keys_lds[slot_of(t)] = key_of(v[u]);
      }
    }
    __syncthreads();
  }
  auto key_at = [&](int t) -> uint32_t { return STAGED ? keys_lds[slot_of(t)] : key_of(m[t]); };

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

  // ---- 1. radix select, most significant digit first: digits of 12, 8, 8 and 4 bits.  The
  //      first digit is wide (sign, exponent and three mantissa bits) because importance values
  //      share their leading bits: with an 8-bit digit most lanes of a wave would hit the same
  //      counter and the LDS would serialise them.  Every boundary shares the empty prefix in
  //      the first pass (one histogram); later passes count only keys that match a boundary's
  //      prefix, which are few.
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = pass == 0 ? 20 : (pass == 1 ? 12 : (pass == 2 ? 4 : 0));
    const int width = pass == 0 ? 12 : (pass == 3 ? 4 : 8);
    const uint32_t dmask = (1u << width) - 1u;
    if (pass == 0) {
      for (int i = tid; i < 4096; i += kThreads) hist0[i] = 0u;
      if (tid < 128) mark[tid] = 0u;
    } else {
      for (int i = tid; i < (kMaxF - 1) * 256; i += kThreads) (&hist[0][0])[i] = 0u;
    }
    __syncthreads();
    uint32_t pre[kMaxF - 1];
#pragma unroll
    for (int g = 0; g < kMaxF - 1; ++g) pre[g] = s_prefix[g];
    for (int t = tid; t < T; t += kThreads) {
      const uint32_t key = key_at(t);
      const uint32_t dig = (key >> shift) & dmask;
      if (pass == 0) {
        atomicAdd(&hist0[dig], 1u);
      } else if ((mark[key >> 25] >> ((key >> 20) & 31u)) & 1u) {
        // one key in hundreds shares its first digit with a boundary; the rest stop here
        const uint32_t hi = key >> (shift + width);
#pragma unroll
        for (int g = 0; g < kMaxF - 1; ++g) {
          if (active[g] && hi == (pre[g] >> (shift + width))) atomicAdd(&hist[g][dig], 1u);
        }
      }
    }
    __syncthreads();
    // wave g walks boundary g's histogram from the top: lane l owns `per` consecutive digits
    bool act_w = false;
#pragma unroll
    for (int g = 0; g < kMaxF - 1; ++g) act_w = act_w || (w == g && active[g]);
    if (act_w) {
      const uint32_t* h = pass == 0 ? hist0 : hist[w];
      const int nbins = 1 << width;
      const int per = nbins >= 64 ? nbins >> 6 : 1;
      const int d0 = lane * per;
      uint32_t tot = 0;
      if (d0 < nbins)
        for (int j = 0; j < per; ++j) tot += h[d0 + j];
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
        for (int j = per - 1; j >= 0; --j) {
          const uint32_t c = h[d0 + j];
          if (k <= acc + c) { digit = (uint32_t)(d0 + j); left = k - acc; break; }
          acc += c;
        }
        s_prefix[w] = s_prefix[w] | (digit << shift);
        s_need[w] = left;
        if (pass == 0) atomicOr(&mark[digit >> 5], 1u << (digit & 31u));
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
  block_excl_scan_n<kMaxF - 1>(eq, wave_tot);               // now: equal keys before t0
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
    if (STAGED) keys_lds[slot_of(t)] = (uint32_t)grp;       // the key is not needed again
    else rank_row[t] = grp;                                 // group id for now, rank below
#pragma unroll
    for (int g = 0; g < kMaxF; ++g) cnt[g] += (grp == g) ? 1 : 0;
  }

  // ---- 3. slot inside the group's ascending index list
  block_excl_scan_n<kMaxF>(cnt, wave_tot);
  int32_t* idx_row = p.bucket_idx + (size_t)b * T;
  for (int t = t0; t < t1; ++t) {
    const int grp = STAGED ? (int)keys_lds[slot_of(t)] : rank_row[t];
    int slot = 0, rk = 0;
#pragma unroll
    for (int g = 0; g < kMaxF; ++g) {
      if (grp == g) { slot = p.bound[g] + cnt[g]; rk = p.grank[g]; cnt[g] += 1; }
    }
    if (!STAGED) rank_row[t] = rk;
    if (slot < T) idx_row[slot] = t;    // always true; keeps a logic error inside the buffer
  }
  if (STAGED) {                         // ranks out, consecutive threads to consecutive tokens
    __syncthreads();
    for (int t = tid; t < T; t += kThreads) {
      const int grp = (int)keys_lds[slot_of(t)];
      int rk = 0;
#pragma unroll
      for (int g = 0; g < kMaxF; ++g) rk = grp == g ? p.grank[g] : rk;
      rank_row[t] = rk;
    }
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
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (kStagedMax + kStagedMax / 32 + 1) * 4);
      if (e != hipSuccess) {
        set_error("hipFuncSetAttribute: %s", hipGetErrorString(e));
        return AP_ERR_HIP;
      }
      attr_set = true;
    }
    hipLaunchKernelGGL(select_ranks_kernel<true>, dim3(B), dim3(kThreads), ((size_t)T + T / 32 + 1) * 4,
                       stream, p);
  } else {
    hipLaunchKernelGGL(select_ranks_kernel<false>, dim3(B), dim3(kThreads), 0, stream, p);
  }
  return check_launch("ap_select_ranks");
}

}  // namespace ap
