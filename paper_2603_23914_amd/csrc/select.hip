// Attention-aware rank groups (paper Sec. 3.2; Alg. 1, group-selection step).
//
// Per batch row the tokens are ordered by (importance descending, token index ascending)
// and cut at fixed sorted positions into F groups.  Nothing is sorted: a group boundary at
// sorted position p is fully described by the p-th largest key kappa and by how many of the
// tokens whose key equals kappa still fall in front of it (the quota), so
//   1. a radix select finds (kappa, quota) of all F-1 boundaries at once (four passes over
//      the row with digits of 12, 8, 8 and 4 bits, histograms in LDS; when few keys share the
//      boundaries' first digits, the last three passes give way to a bit-by-bit search over
//      those few keys in registers);
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
#include "lane_ops.hpp"

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
#ifdef AP_KERNEL_TIMERS
  unsigned long long* stamps;   // kernel studies: 16 time stamps of row 0's first and last thread (100 MHz counter)
#endif
};

#ifdef AP_KERNEL_TIMERS
#define AP_SELECT_STAMP(i) do { if (blockIdx.x == 0 && (threadIdx.x == 0 || threadIdx.x == 1023)) p.stamps[(threadIdx.x ? 16 : 0) + (i)] = wall_clock64(); } while (0)
#else
#define AP_SELECT_STAMP(i) do { } while (0)
#endif

// Order-preserving map float -> uint32 (larger value, larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t key_of(float m) {
  uint32_t u = __builtin_bit_cast(uint32_t, m);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sums over the workgroup (thread order) of the first n of N values per thread
// at once (two barriers for all of them; n is the same for every thread, v[k] stays as it is
// for k >= n).  wave_tot: N * kWaves ints.
template <int N>
__device__ __forceinline__ void block_excl_scan_n(int (&v)[N], int n, int* wave_tot) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl[N];
#pragma unroll
  for (int k = 0; k < N; ++k) incl[k] = v[k];
#pragma unroll
  for (int k = 0; k < N; ++k) {
    if (k < n) {
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl[k], o);
        if (lane >= o) incl[k] += up;
      }
    }
  }
  __syncthreads();                       // previous use of wave_tot is over
  if (lane == 63) {
#pragma unroll
    for (int k = 0; k < N; ++k)
      if (k < n) wave_tot[k * kWaves + w] = incl[k];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < N; ++k) {
    if (k < n) {
      int base = 0;
#pragma unroll
      for (int i = 0; i < kWaves; ++i) {
        const int x = wave_tot[k * kWaves + i];
        if (i < w) base += x;
      }
      v[k] = base + incl[k] - v[k];
    }
  }
}

constexpr int kCand = 256;             // candidate keys per boundary that the short cut after the first pass takes
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
  __shared__ uint32_t s_ncand[kMaxF - 1];    // short cut after the first pass: candidates listed so far
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int b = blockIdx.x, T = p.T, F = p.F, nb = F - 1;
  const float* m = p.mass + (size_t)b * T;
  AP_SELECT_STAMP(0);
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
  AP_SELECT_STAMP(1);

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
    s_ncand[tid] = 0u;
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
          if (g < nb && active[g] && hi == (pre[g] >> (shift + width))) atomicAdd(&hist[g][dig], 1u);
        }
      }
    }
    __syncthreads();
    AP_SELECT_STAMP(2 + 2 * pass);
    // wave g walks boundary g's histogram from the top: lane l owns `per` consecutive digits
    bool act_w = false;
#pragma unroll
    for (int g = 0; g < kMaxF - 1; ++g) act_w = act_w || (w == g && active[g]);
    if (act_w) {
      const uint32_t* h = pass == 0 ? hist0 : hist[w];
      const int nbins = 1 << width;
      const int per = nbins >= 64 ? nbins >> 6 : 1;          // 64, 4, 4, 1: a power of two
      auto suffix = [&](uint32_t v) -> uint32_t {            // sum over lanes >= lane
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const uint32_t dn = (uint32_t)__shfl_down((int)v, o);
          if (lane + o < 64) v += dn;
        }
        return v;
      };
      // first level: lane l sums its `per` consecutive digits (read in an order rotated by the
      // lane, so the lanes of a wave touch different banks) ...
      const int d0 = lane * per;
      uint32_t tot = 0;
      if (pass == 0) {                                       // 64 loads in flight, then one sum
        uint32_t c64[64];
#pragma unroll
        for (int j = 0; j < 64; ++j) c64[j] = h[d0 + ((j + lane) & 63)];
#pragma unroll
        for (int j = 0; j < 64; ++j) tot += c64[j];
      } else if (d0 < nbins) {
        for (int j = 0; j < per; ++j) tot += h[d0 + ((j + lane) & (per - 1))];
      }
      const uint32_t incl = suffix(tot);
      const uint32_t above = incl - tot;
      const uint32_t k = s_need[w];
      const unsigned long long owner = __ballot(above < k && k <= incl);   // exactly one lane
      if (owner) {
        // ... second level: the digits of the owning lane's block, one per lane
        const int L = __ffsll(owner) - 1;
        const uint32_t k2 = k - (uint32_t)__shfl((int)above, L);
        const uint32_t c = lane < per ? h[L * per + lane] : 0u;
        const uint32_t incl2 = suffix(c);
        const uint32_t above2 = incl2 - c;
        if (lane < per && above2 < k2 && k2 <= incl2) {                    // exactly one lane
          const uint32_t digit = (uint32_t)(L * per + lane);
          s_prefix[w] = s_prefix[w] | (digit << shift);
          s_need[w] = k2 - above2;
          if (pass == 0) atomicOr(&mark[digit >> 5], 1u << (digit & 31u));
        }
      }
    }
    __syncthreads();
    AP_SELECT_STAMP(3 + 2 * pass);
    if (pass == 0) {
      // ---- short cut: when at most kCand keys share the first digit of every boundary (the
      //      usual case: one key in hundreds does), the remaining 20 bits are not found by
      //      three more histogram passes.  The few candidate keys of a boundary are listed in
      //      LDS (in the space of its later histograms), its wave takes them into registers and
      //      fixes the 20 bits one at a time, counting with wave-wide ballots.
      bool few = true;
#pragma unroll
      for (int g = 0; g < kMaxF - 1; ++g)
        if (g < nb && active[g]) few = few && hist0[s_prefix[g] >> 20] <= (uint32_t)kCand;
      if (few) {
        uint32_t dig[kMaxF - 1];
#pragma unroll
        for (int g = 0; g < kMaxF - 1; ++g) dig[g] = s_prefix[g] >> 20;
        for (int t = tid; t < T; t += kThreads) {
          const uint32_t key = key_at(t);
          if ((mark[key >> 25] >> ((key >> 20) & 31u)) & 1u) {
#pragma unroll
            for (int g = 0; g < kMaxF - 1; ++g) {
              if (g < nb && active[g] && (key >> 20) == dig[g]) {
                const uint32_t at = atomicAdd(&s_ncand[g], 1u);
                if (at < (uint32_t)kCand) hist[g][at] = key & 0xfffffu;   // always true: the count was checked
              }
            }
          }
        }
        __syncthreads();
        if (act_w) {
          const uint32_t n = hist0[s_prefix[w] >> 20];
          uint32_t c[kCand / 64];
          bool have[kCand / 64];
#pragma unroll
          for (int k = 0; k < kCand / 64; ++k) {
            have[k] = (uint32_t)(lane + 64 * k) < n;
            c[k] = have[k] ? hist[w][lane + 64 * k] : 0u;
          }
          uint32_t low = 0u, need = s_need[w];
          for (int bit = 19; bit >= 0; --bit) {
            const uint32_t trial = (low | (1u << bit)) >> bit;   // the bits above `bit` as fixed, this one set
            uint32_t n1 = 0;
#pragma unroll
            for (int k = 0; k < kCand / 64; ++k) n1 += (uint32_t)__popcll(__ballot(have[k] && (c[k] >> bit) == trial));
            if (need <= n1) low |= 1u << bit;                     // the wanted key has this bit set
            else need -= n1;                                      // all of those lie in front of it
          }
          if (lane == 0) {
            s_prefix[w] = s_prefix[w] | low;
            s_need[w] = need;
          }
        }
        __syncthreads();
        AP_SELECT_STAMP(9);
        break;
      }
    }
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
    for (int g = 0; g < kMaxF - 1; ++g)
      if (g < nb) eq[g] += (key == kappa[g]) ? 1 : 0;       // nb is the same for all: a scalar branch
  }
  AP_SELECT_STAMP(10);
  block_excl_scan_n<kMaxF - 1>(eq, nb, wave_tot);               // now: equal keys before t0
  AP_SELECT_STAMP(11);
  int cnt[kMaxF];
#pragma unroll
  for (int g = 0; g < kMaxF; ++g) cnt[g] = 0;
  int32_t* rank_row = p.rank_out + (size_t)b * T;
  for (int t = t0; t < t1; ++t) {
    const uint32_t key = key_at(t);
    int grp = nb;
#pragma unroll
    for (int g = kMaxF - 2; g >= 0; --g) {
      if (g < nb) {
        const bool same = key == kappa[g];
        const bool in_front = key > kappa[g] || (same && (uint32_t)eq[g] < quota[g]);
        if (in_front) grp = g;                              // membership is nested: keep the smallest
        eq[g] += same ? 1 : 0;
      }
    }
    if (STAGED) keys_lds[slot_of(t)] = (uint32_t)grp;       // the key is not needed again
    else rank_row[t] = grp;                                 // group id for now, rank below
#pragma unroll
    for (int g = 0; g < kMaxF; ++g)
      if (g < F) cnt[g] += (grp == g) ? 1 : 0;
  }

  // ---- 3. slot inside the group's ascending index list
  AP_SELECT_STAMP(12);
  block_excl_scan_n<kMaxF>(cnt, F, wave_tot);
  AP_SELECT_STAMP(13);
  int32_t* idx_row = p.bucket_idx + (size_t)b * T;
  for (int t = t0; t < t1; ++t) {
    const int grp = STAGED ? (int)keys_lds[slot_of(t)] : rank_row[t];
    int slot = 0, rk = 0;
#pragma unroll
    for (int g = 0; g < kMaxF; ++g) {
      if (g < F && grp == g) { slot = p.bound[g] + cnt[g]; rk = p.grank[g]; cnt[g] += 1; }
    }
    if (!STAGED) rank_row[t] = rk;
    if (slot < T) idx_row[slot] = t;    // always true; keeps a logic error inside the buffer
  }
  AP_SELECT_STAMP(14);
  if (STAGED) {                         // ranks out, consecutive threads to consecutive tokens
    __syncthreads();
    for (int t = tid; t < T; t += kThreads) {
      const int grp = (int)keys_lds[slot_of(t)];
      int rk = 0;
#pragma unroll
      for (int g = 0; g < kMaxF; ++g)
        if (g < F) rk = grp == g ? p.grank[g] : rk;
      rank_row[t] = rk;
    }
  }
  int cut = 0;
#pragma unroll
  for (int g = 0; g <= kMaxF; ++g) cut = tid == g ? p.bound[g] : cut;
  if (tid <= F) p.bucket_off[(size_t)b * (F + 1) + tid] = cut;
  AP_SELECT_STAMP(15);
}

// Importance update of Eq. 1 for one new query: the attention weights of the query, averaged
// over the heads, enter the moving average.  scores [B][T_cap][H]: the H logits of a token are
// contiguous.
//
// update_importance_rows (H a multiple of 4, at most 256, 16-byte aligned pointers): grid
// (ceil(T / 128), B), 256 threads.  A workgroup's 128 tokens are one contiguous run of 128 H
// logits; thread i takes the i-th 16-byte word of it (four heads of one token), turns it into
// the sum of four weights and leaves that in LDS; one thread per token then adds the token's
// H / 4 partial sums in head order.
constexpr int kImpTokens = 128;
constexpr int kImpMaxH = 256;
__global__ void __launch_bounds__(256)
update_importance_rows(const float* __restrict__ scores, const float* __restrict__ lse,
                       float* __restrict__ mass, int H, int T, int T_cap, int64_t mass_stride,
                       float alpha) {
  extern __shared__ float part[];                // [128 tokens][H / 4]
  const int tid = threadIdx.x, b = blockIdx.y;
  const int t0 = blockIdx.x * kImpTokens;
  int nt = T - t0;
  nt = nt < kImpTokens ? nt : kImpTokens;
  const int H4 = H >> 2, n4 = nt * H4;
  const f32x4_t* s4 = (const f32x4_t*)(scores + ((size_t)b * T_cap + t0) * H);
  const f32x4_t* l4 = (const f32x4_t*)(lse + (size_t)b * H);
  const float inv_h4 = 1.0f / (float)H4;         // i / H4 below: exact, i < 2^14
  float* m = mass + (size_t)b * mass_stride + t0 + tid;
  const float m_old = tid < nt ? *m : 0.f;       // asked for early, needed last
  for (int i0 = tid; i0 < n4; i0 += 256 * 4) {   // four 16-byte loads in flight per thread
    f32x4_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = i0 + 256 * k < n4 ? s4[i0 + 256 * k] : f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + 256 * k;
      if (i < n4) {
        const f32x4_t l = l4[i - (int)(((float)i + 0.5f) * inv_h4) * H4];
        part[i] = (__expf(v[k][0] - l[0]) + __expf(v[k][1] - l[1])) + (__expf(v[k][2] - l[2]) + __expf(v[k][3] - l[3]));
      }
    }
  }
  __syncthreads();
  if (tid < nt) {
    float acc = 0.f;
    for (int j = 0; j < H4; ++j) acc += part[tid * H4 + j];
    *m = alpha * m_old + (1.0f - alpha) * (acc / (float)H);
  }
}

// Any H: one thread per token walks the token's H logits.  grid (ceil(T / 256), B).
__global__ void __launch_bounds__(256)
update_importance_any(const float* __restrict__ scores, const float* __restrict__ lse,
                      float* __restrict__ mass, int H, int T, int T_cap, int64_t mass_stride,
                      float alpha) {
  const int t = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
  if (t >= T) return;
  const float* s = scores + ((size_t)b * T_cap + t) * H;
  const float* l = lse + (size_t)b * H;
  float acc = 0.f;
  for (int h = 0; h < H; ++h) acc += __expf(s[h] - l[h]);
  float* m = mass + (size_t)b * mass_stride + t;
  *m = alpha * *m + (1.0f - alpha) * (acc / (float)H);
}

}  // namespace

ap_status launch_update_importance(const float* scores, const float* lse, float* mass, int B, int H,
                                   int T, int T_cap, int64_t mass_stride, float alpha,
                                   hipStream_t stream) {
  const bool rows = (H & 3) == 0 && H <= kImpMaxH && (((uintptr_t)scores | (uintptr_t)lse) & 15) == 0;
  if (rows) {
    hipLaunchKernelGGL(update_importance_rows, dim3((T + kImpTokens - 1) / kImpTokens, B), dim3(256),
                       (size_t)kImpTokens * H, stream, scores, lse, mass, H, T, T_cap, mass_stride, alpha);
  } else {
    hipLaunchKernelGGL(update_importance_any, dim3((T + 255) / 256, B), dim3(256), 0, stream, scores, lse,
                       mass, H, T, T_cap, mass_stride, alpha);
  }
  return check_launch("ap_update_importance");
}

size_t select_workspace(int, int, int) { return 256; }   // every intermediate lives in LDS

ap_status launch_select_ranks(const float* mass, int B, int T, int F, const int32_t* group_rank,
                              const int32_t* cum_num, int32_t den, int32_t* rank_out,
                              int32_t* bucket_off, int32_t* bucket_idx, void* ws,
                              hipStream_t stream) {
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
#ifdef AP_KERNEL_TIMERS
  p.stamps = (unsigned long long*)ws;
#else
  (void)ws;
#endif
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
