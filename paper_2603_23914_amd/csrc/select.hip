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
// pass.  All integer work, results are unique.  Few, long rows take the same steps with a row
// split over workgroups (the split_* kernels below).
#include "ap_common.hpp"
#include "lane_ops.hpp"

#include <cstdlib>
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
  uint32_t* split_ws;         // rows split over workgroups: per-row scratch (see SplitLayout), else null
  int per;                    // ... and the tokens each thread owns there
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
// for k >= n).  NW waves per workgroup; wave_tot: N * NW ints.
template <int N, int NW = kWaves>
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
      if (k < n) wave_tot[k * NW + w] = incl[k];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < N; ++k) {
    if (k < n) {
      int base = 0;
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        const int x = wave_tot[k * NW + i];
        if (i < w) base += x;
      }
      v[k] = base + incl[k] - v[k];
    }
  }
}

constexpr int kCand = 256;             // candidate keys per boundary that the short cut after the first pass takes
constexpr int kStagedMax = 32768;      // tokens whose keys fit the dynamic LDS slice (132 KiB with padding)

// Rows split over workgroups (long rows, few of them): a workgroup of 256 threads owns a chunk of
// 256 * per consecutive tokens, a thread `per` consecutive ones.  Per-row scratch in the caller's
// workspace, in 32-bit words:
//   hist   [G][4096]  first-digit histogram of every chunk
//   ctl    [64]       candidate counters, the gave-up flag, and per boundary: first digit, position
//                     still to find
//   cand   [7][cap]   low 20 key bits of the keys that share a boundary's first digit
//   candt  [7][cap]   their token indices (cap: an eighth of the row, at least 4096)
//   counts [G][8]     tokens of every group in every chunk
constexpr int kSplitThreads = 256;
constexpr int kSplitWaves = kSplitThreads / 64;
constexpr int kSplitMaxChunks = 64;
constexpr int kEqMax = 256;            // tokens per boundary that may share kappa itself
constexpr int kStage = 2048;           // candidates of a boundary that are walked from LDS
constexpr int kSplitMinT = 24576;      // rows at least this long ...
constexpr int kSplitMaxB = 32;         // ... in batches of at most this many rows, or rows beyond kStagedMax
constexpr int kCtlNcand = 0, kCtlGaveUp = 7, kCtlDigit = 8, kCtlNeed = 16;
struct SplitLayout {
  int G, cap;
  size_t hist, ctl, cand, candt, counts, stride;
};
__host__ __device__ inline SplitLayout split_layout(int T, int per) {
  SplitLayout L;
  const int chunk = kSplitThreads * per;
  L.G = (T + chunk - 1) / chunk;
  L.hist = 0;
  L.ctl = L.hist + (size_t)L.G * 4096;
  L.cap = T / 8 < 4096 ? 4096 : (T / 8 + 63) / 64 * 64;
  L.cand = L.ctl + 64;
  L.candt = L.cand + (size_t)(kMaxF - 1) * L.cap;
  L.counts = L.candt + (size_t)(kMaxF - 1) * L.cap;
  L.stride = L.counts + (size_t)L.G * kMaxF;
  return L;
}
// tokens per thread: eight, or as many as keep a row within kSplitMaxChunks chunks
inline int split_per(int T) {
  const int per = (T + kSplitThreads * kSplitMaxChunks - 1) / (kSplitThreads * kSplitMaxChunks);
  return per < 8 ? 8 : (per + 7) / 8 * 8;
}

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
  // after the split kernels: only the rows they gave up on (too many keys share a boundary's
  // leading bits) are done here
  if (p.split_ws && p.split_ws[split_layout(T, p.per).stride * b + split_layout(T, p.per).ctl + kCtlGaveUp] == 0u) return;
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


// ------------------------------------------------------------------------------------------
// The same selection with a row split over workgroups, for batches too small to fill the chip
// with one workgroup per row.  Four launches over grid (G chunks, B rows), 256 threads:
//   split_hist    first-digit (12-bit) histogram of every chunk, to the workspace;
//   split_cand    every workgroup adds the chunks' histograms up, finds each boundary's first
//                 digit, and lists the keys of its chunk that share it (with their tokens);
//   split_groups  every workgroup fixes the other 20 bits of each boundary's kappa from that
//                 list (a wave per boundary, digits of 8, 8 and 4 bits), notes the tokens whose
//                 key is kappa itself, gives its tokens their groups and counts them; a token
//                 whose key equals kappa finds its position among the equal keys by counting the
//                 noted tokens in front of it;
//   split_emit    prefix sums of the chunks' group counts place every token in its group's
//                 ascending index list.
// A row where more than an eighth of the keys share a boundary's first digit, or more than
// kEqMax tokens a boundary's kappa, raises a flag instead, and the one-workgroup kernel,
// launched after these, does exactly the flagged rows.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_suffix_sum(uint32_t v) {     // sum over lanes >= lane
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t dn = (uint32_t)__shfl_down((int)v, o);
    if (lane + o < 64) v += dn;
  }
  return v;
}
// One wave finds the digit that holds the k-th largest entry (1-based) of a histogram of NBINS
// counters (4096 or 256), and the position left inside that digit.  False when k exceeds the total.
template <int NBINS>
__device__ __forceinline__ bool walk_digit(const uint32_t* h, uint32_t k, uint32_t& digit, uint32_t& rest) {
  constexpr int per = NBINS / 64;
  const int lane = threadIdx.x & 63;
  uint32_t tot = 0;
  for (int j = 0; j < per; ++j) tot += h[lane * per + ((j + lane) & (per - 1))];
  const uint32_t incl = wave_suffix_sum(tot), above = incl - tot;
  const unsigned long long owner = __ballot(above < k && k <= incl);
  if (!owner) return false;
  const int L = __ffsll(owner) - 1;
  const uint32_t k2 = k - (uint32_t)__shfl((int)above, L);
  const uint32_t c = lane < per ? h[L * per + lane] : 0u;
  const uint32_t incl2 = wave_suffix_sum(c), above2 = incl2 - c;
  const unsigned long long hit = __ballot(lane < per && above2 < k2 && k2 <= incl2);
  if (!hit) return false;
  const int Hh = __ffsll(hit) - 1;
  digit = (uint32_t)(L * per + Hh);
  rest = k2 - (uint32_t)__shfl((int)above2, Hh);
  return true;
}

struct SplitParams {
  const float* mass;
  uint32_t* ws;
  int T, F, per;
  int32_t bound[kMaxF + 1];
  int32_t grank[kMaxF];
  int32_t* rank_out;
  int32_t* bucket_off;
  int32_t* bucket_idx;
};

// eight of a thread's keys at once (tokens t .. t + 7, those at or beyond t1 read as token t1 - 1)
__device__ __forceinline__ void load_keys8(const float* m, int t, int t1, uint32_t (&k)[8]) {
  float v[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) v[u] = m[t + u < t1 ? t + u : t1 - 1];
#pragma unroll
  for (int u = 0; u < 8; ++u) k[u] = key_of(v[u]);
}

__global__ void __launch_bounds__(kSplitThreads) split_hist(const SplitParams p) {
  __shared__ uint32_t h[4096];
  const int tid = threadIdx.x, c = blockIdx.x, b = blockIdx.y, T = p.T;
  const SplitLayout L = split_layout(T, p.per);
  uint32_t* ws = p.ws + L.stride * b;
  for (int i = tid; i < 4096; i += kSplitThreads) h[i] = 0u;
  if (c == 0 && tid < 8) ws[L.ctl + tid] = 0u;                // candidate counters and the flag
  __syncthreads();
  const float* m = p.mass + (size_t)b * T;
  const int t0 = min(T, (c * kSplitThreads + tid) * p.per), t1 = min(T, t0 + p.per);
  for (int t = t0; t < t1; t += 8) {
    uint32_t k[8];
    load_keys8(m, t, t1, k);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (t + u < t1) atomicAdd(&h[k[u] >> 20], 1u);
  }
  __syncthreads();
  uint32_t* dst = ws + L.hist + (size_t)c * 4096;
  for (int i = tid; i < 4096; i += kSplitThreads) dst[i] = h[i];
}

__global__ void __launch_bounds__(kSplitThreads) split_cand(const SplitParams p) {
  __shared__ __attribute__((aligned(16))) uint32_t h[4096];
  __shared__ uint32_t s_digit[kMaxF - 1], s_need[kMaxF - 1];
  __shared__ uint32_t s_cnt[kMaxF - 1], s_cnt2[kMaxF - 1], s_base[kMaxF - 1];
  __shared__ int s_few;
  const int tid = threadIdx.x, w = tid >> 6, c = blockIdx.x, b = blockIdx.y, T = p.T, nb = p.F - 1;
  const SplitLayout L = split_layout(T, p.per);
  uint32_t* ws = p.ws + L.stride * b;
  // the row's histogram: sixteen counters per thread (four 16-byte words), the chunks' copies
  // summed, eight chunks' loads in flight at a time
  {
    u32x4_t acc[4];
    const u32x4_t zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = zero;
    const u32x4_t* src = (const u32x4_t*)(ws + L.hist) + tid;
    for (int g0 = 0; g0 < L.G; g0 += 8) {
      u32x4_t v[8][4];
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          v[k][i] = g0 + k < L.G ? src[(size_t)(g0 + k) * 1024 + i * kSplitThreads] : zero;
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] += v[k][i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) *(u32x4_t*)&h[(i * kSplitThreads + tid) * 4] = acc[i];
  }
  if (tid == 0) s_few = 1;
  if (tid < kMaxF - 1) { s_digit[tid] = kNone; s_need[tid] = 0u; s_cnt[tid] = 0u; s_cnt2[tid] = 0u; s_base[tid] = 0u; }
  __syncthreads();
  for (int g = w; g < nb; g += kSplitWaves) {                 // a wave per boundary
    const int cut = p.bound[g + 1];
    if (cut > 0 && cut < T) {
      uint32_t digit = 0u, rest = 0u;
      const bool ok = walk_digit<4096>(h, (uint32_t)cut, digit, rest);
      if ((tid & 63) == 0) {
        if (!ok || h[digit] > (uint32_t)L.cap) s_few = 0;
        else { s_digit[g] = digit; s_need[g] = rest; }
      }
    }
  }
  __syncthreads();
  if (!s_few) {
    if (c == 0 && tid == 0) ws[L.ctl + kCtlGaveUp] = 1u;
    return;
  }
  uint32_t dig[kMaxF - 1];
#pragma unroll
  for (int g = 0; g < kMaxF - 1; ++g) dig[g] = s_digit[g];     // kNone: no key has that first digit
  if (c == 0 && tid < kMaxF - 1) {
    ws[L.ctl + kCtlDigit + tid] = s_digit[tid];
    ws[L.ctl + kCtlNeed + tid] = s_need[tid];
  }
  // the chunk's candidates are counted first, so that one addition per boundary reserves their
  // places in the row's lists; the order inside a list is immaterial
  const float* m = p.mass + (size_t)b * T;
  const int t0 = min(T, (c * kSplitThreads + tid) * p.per), t1 = min(T, t0 + p.per);
  for (int t = t0; t < t1; t += 8) {
    uint32_t k[8];
    load_keys8(m, t, t1, k);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (t + u < t1) {
#pragma unroll
        for (int g = 0; g < kMaxF - 1; ++g)
          if ((k[u] >> 20) == dig[g]) atomicAdd(&s_cnt[g], 1u);
      }
    }
  }
  __syncthreads();
  if (tid < kMaxF - 1 && s_cnt[tid]) s_base[tid] = atomicAdd(&ws[L.ctl + kCtlNcand + tid], s_cnt[tid]);
  __syncthreads();
  for (int t = t0; t < t1; t += 8) {
    uint32_t k[8];
    load_keys8(m, t, t1, k);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (t + u < t1) {
#pragma unroll
        for (int g = 0; g < kMaxF - 1; ++g) {
          if ((k[u] >> 20) == dig[g]) {
            const uint32_t at = s_base[g] + atomicAdd(&s_cnt2[g], 1u);
            if (at < (uint32_t)L.cap) {                        // always true: the count was checked
              ws[L.cand + (size_t)g * L.cap + at] = k[u] & 0xfffffu;
              ws[L.candt + (size_t)g * L.cap + at] = (uint32_t)(t + u);
            }
          }
        }
      }
    }
  }
}

// The group of a token: the first boundary it lies in front of (membership is nested).  A token
// whose key equals a boundary's kappa counts the listed tokens with that key in front of it.
__device__ __forceinline__ int group_of(uint32_t key, int t, int nb, const uint32_t (&kappa)[kMaxF - 1],
                                        const uint32_t (&quota)[kMaxF - 1], const uint32_t* s_eq,
                                        const uint32_t* s_neq) {
  int grp = nb;
#pragma unroll
  for (int g = kMaxF - 2; g >= 0; --g) {
    if (g < nb) {
      bool in_front = key > kappa[g];
      if (key == kappa[g]) {
        uint32_t pos = 0;
        const uint32_t n = s_neq[g];
        for (uint32_t i = 0; i < n; ++i) pos += s_eq[g * kEqMax + i] < (uint32_t)t ? 1u : 0u;
        in_front = pos < quota[g];
      }
      if (in_front) grp = g;
    }
  }
  return grp;
}

__global__ void __launch_bounds__(kSplitThreads) split_groups(const SplitParams p) {
  __shared__ uint32_t hw[kSplitWaves][256];                    // a histogram per wave
  __shared__ uint32_t s_cl[kSplitWaves][kStage];               // ... and its boundary's candidates
  __shared__ uint32_t s_eq[(kMaxF - 1) * kEqMax];              // tokens whose key equals kappa
  __shared__ uint32_t s_neq[kMaxF - 1], s_kappa[kMaxF - 1], s_quota[kMaxF - 1];
  __shared__ int s_cnt[kMaxF];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int c = blockIdx.x, b = blockIdx.y, T = p.T, F = p.F, nb = F - 1;
  const SplitLayout L = split_layout(T, p.per);
  uint32_t* ws = p.ws + L.stride * b;
  if (ws[L.ctl + kCtlGaveUp]) return;
  if (tid < kMaxF) s_cnt[tid] = 0;
  if (tid < kMaxF - 1) {
    const int cut = tid < nb ? p.bound[tid + 1] : 0;
    s_neq[tid] = 0u;
    // a cut at 0: nobody in front; a cut at T: everybody
    s_kappa[tid] = (tid < nb && cut >= T) ? 0u : kNone;
    s_quota[tid] = (tid < nb && cut >= T) ? (uint32_t)T : 0u;
  }
  __syncthreads();
  for (int g = w; g < nb; g += kSplitWaves) {
    // a wave per boundary: the other 20 bits of kappa, by digits of 8, 8 and 4 bits over the
    // boundary's candidate list
    const int cut = p.bound[g + 1];
    if (cut > 0 && cut < T) {
      const uint32_t n = min(ws[L.ctl + kCtlNcand + g], (uint32_t)L.cap);
      const uint32_t* cl = ws + L.cand + (size_t)g * L.cap;
      const uint32_t* ct = ws + L.candt + (size_t)g * L.cap;
      uint32_t low = 0u, need = ws[L.ctl + kCtlNeed + g];
      const uint32_t digit1 = ws[L.ctl + kCtlDigit + g];
      bool ok = true;
      auto resolve = [&](auto cand_at) {
#pragma unroll 1
        for (int pass = 0; pass < 3; ++pass) {
          const int shift = pass == 0 ? 12 : (pass == 1 ? 4 : 0);
          const int width = pass == 2 ? 4 : 8;
          // the wave's own histogram: its LDS operations complete in program order
          for (int i = lane; i < 256; i += 64) hw[w][i] = 0u;
          __builtin_amdgcn_wave_barrier();
          for (uint32_t i0 = lane; i0 < n; i0 += 512) {          // eight loads in flight
            uint32_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = i0 + 64 * u < n ? cand_at(i0 + 64 * u) : 0u;
#pragma unroll
            for (int u = 0; u < 8; ++u)
              if (i0 + 64 * u < n && (v[u] >> (shift + width)) == (low >> (shift + width)))
                atomicAdd(&hw[w][(v[u] >> shift) & ((1u << width) - 1u)], 1u);
          }
          __builtin_amdgcn_wave_barrier();
          uint32_t digit = 0u, rest = 0u;
          ok = ok && walk_digit<256>(hw[w], need, digit, rest);
          low |= digit << shift;
          need = rest;
        }
        for (uint32_t i0 = lane; i0 < n; i0 += 512) {
          uint32_t v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) v[u] = i0 + 64 * u < n ? cand_at(i0 + 64 * u) : kNone;
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            if (v[u] == low) {                                   // kNone is no 20-bit value
              const uint32_t at = atomicAdd(&s_neq[g], 1u);
              if (at < (uint32_t)kEqMax) s_eq[g * kEqMax + at] = ct[i0 + 64 * u];
            }
          }
        }
      };
      if (n <= (uint32_t)kStage) {
        // a list this short moves to LDS first (sixteen loads in flight): the four walks over it
        // then cost no trips to memory
        for (uint32_t i0 = lane; i0 < n; i0 += 1024) {
          uint32_t v[16];
#pragma unroll
          for (int u = 0; u < 16; ++u) v[u] = i0 + 64 * u < n ? cl[i0 + 64 * u] : 0u;
#pragma unroll
          for (int u = 0; u < 16; ++u)
            if (i0 + 64 * u < n) s_cl[w][i0 + 64 * u] = v[u];
        }
        __builtin_amdgcn_wave_barrier();
        resolve([&](uint32_t i) { return s_cl[w][i]; });
      } else {
        resolve([&](uint32_t i) { return cl[i]; });
      }
      if (lane == 0) {
        s_kappa[g] = (digit1 << 20) | low;
        s_quota[g] = need;
        if (!ok) s_neq[g] = kEqMax + 1;                        // cannot happen; treated as giving up
      }
    }
  }
  __syncthreads();
  bool fits = true;
#pragma unroll
  for (int g = 0; g < kMaxF - 1; ++g) fits = fits && s_neq[g] <= (uint32_t)kEqMax;
  if (!fits) {                                                 // every workgroup of the row sees the same
    if (c == 0 && tid == 0) ws[L.ctl + kCtlGaveUp] = 1u;
    return;
  }
  uint32_t kappa[kMaxF - 1], quota[kMaxF - 1];
#pragma unroll
  for (int g = 0; g < kMaxF - 1; ++g) { kappa[g] = s_kappa[g]; quota[g] = s_quota[g]; }
  const float* m = p.mass + (size_t)b * T;
  int32_t* rank_row = p.rank_out + (size_t)b * T;
  const int t0 = min(T, (c * kSplitThreads + tid) * p.per), t1 = min(T, t0 + p.per);
  int cnt[kMaxF];
#pragma unroll
  for (int g = 0; g < kMaxF; ++g) cnt[g] = 0;
  for (int t = t0; t < t1; t += 8) {
    uint32_t k[8];
    load_keys8(m, t, t1, k);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (t + u < t1) {
        const int grp = group_of(k[u], t + u, nb, kappa, quota, s_eq, s_neq);
        rank_row[t + u] = grp;                                // group id for now, rank in split_emit
#pragma unroll
        for (int g = 0; g < kMaxF; ++g) cnt[g] += (grp == g) ? 1 : 0;
      }
    }
  }
#pragma unroll
  for (int g = 0; g < kMaxF; ++g)
    if (g < F && cnt[g]) atomicAdd(&s_cnt[g], cnt[g]);
  __syncthreads();
  if (tid < kMaxF) ws[L.counts + (size_t)c * kMaxF + tid] = (uint32_t)s_cnt[tid];
}

__global__ void __launch_bounds__(kSplitThreads) split_emit(const SplitParams p) {
  __shared__ int wave_tot[kMaxF * kSplitWaves];
  __shared__ int s_base[kMaxF];
  const int tid = threadIdx.x;
  const int c = blockIdx.x, b = blockIdx.y, T = p.T, F = p.F;
  const SplitLayout L = split_layout(T, p.per);
  const uint32_t* ws = p.ws + L.stride * b;
  if (ws[L.ctl + kCtlGaveUp]) return;
  if (tid < kMaxF) {
    int base = 0;
#pragma unroll
    for (int g = 0; g < kMaxF; ++g) base = tid == g ? p.bound[g] : base;
    for (int k0 = 0; k0 < c; k0 += 8) {                        // eight loads in flight
      uint32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = k0 + u < c ? ws[L.counts + (size_t)(k0 + u) * kMaxF + tid] : 0u;
#pragma unroll
      for (int u = 0; u < 8; ++u) base += (int)v[u];
    }
    s_base[tid] = base;
  }
  int32_t* rank_row = p.rank_out + (size_t)b * T;
  int32_t* idx_row = p.bucket_idx + (size_t)b * T;
  const int t0 = min(T, (c * kSplitThreads + tid) * p.per), t1 = min(T, t0 + p.per);
  int cnt[kMaxF];
#pragma unroll
  for (int g = 0; g < kMaxF; ++g) cnt[g] = 0;
  auto load_groups8 = [&](int t, int (&grp)[8]) {
#pragma unroll
    for (int u = 0; u < 8; ++u) grp[u] = rank_row[t + u < t1 ? t + u : t1 - 1];
  };
  for (int t = t0; t < t1; t += 8) {
    int grp[8];
    load_groups8(t, grp);
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int g = 0; g < kMaxF; ++g) cnt[g] += (t + u < t1 && grp[u] == g) ? 1 : 0;
  }
  block_excl_scan_n<kMaxF, kSplitWaves>(cnt, F, wave_tot);      // its barriers also publish s_base
  for (int t = t0; t < t1; t += 8) {
    int grp[8];
    load_groups8(t, grp);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (t + u < t1) {
        int slot = T, rk = 0;
#pragma unroll
        for (int g = 0; g < kMaxF; ++g) {
          if (g < F && grp[u] == g) { slot = s_base[g] + cnt[g]; rk = p.grank[g]; cnt[g] += 1; }
        }
        rank_row[t + u] = rk;
        if (slot < T) idx_row[slot] = t + u;   // always true; keeps a logic error inside the buffer
      }
    }
  }
  int cut = 0;
#pragma unroll
  for (int g = 0; g <= kMaxF; ++g) cut = tid == g ? p.bound[g] : cut;
  if (c == 0 && tid <= F) p.bucket_off[(size_t)b * (F + 1) + tid] = cut;
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

// One workgroup per row fills the chip when there are many rows, and a short row is done before
// four more launches would be (each hands its results to the next through memory: about 45 us in
// all, whatever the length): the split is for few, long rows (measured at four groups: 32768
// tokens 45-55 us against 92-96, 16384 tokens about even), and for rows too long for the one
// workgroup's LDS copy, which it would otherwise re-read from memory seven times (131072 tokens:
// 61-95 us against 650).
static bool split_applies(int B, int T) {
#ifdef AP_KERNEL_TIMERS
  return false;                          // the stamps live where the split's scratch would
#else
#ifdef AP_SELECT_SPLIT_ENV
  if (const char* e = getenv("AP_SELECT_SPLIT")) return atoi(e) != 0;
#endif
  return T > kStagedMax || (T >= kSplitMinT && B <= kSplitMaxB);
#endif
}
size_t select_workspace(int B, int T, int) {
  // without the split every intermediate lives in LDS
  return split_applies(B, T) ? 256 + (size_t)B * split_layout(T, split_per(T)).stride * 4 : 256;
}

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
  p.split_ws = nullptr;
  p.per = 0;
#ifdef AP_KERNEL_TIMERS
  p.stamps = (unsigned long long*)ws;
#endif
  if (split_applies(B, T)) {
    SplitParams sp;
    sp.mass = mass;
    sp.ws = (uint32_t*)ws;
    sp.T = T;
    sp.F = F;
    sp.per = split_per(T);
    for (int g = 0; g <= kMaxF; ++g) sp.bound[g] = p.bound[g];
    for (int g = 0; g < kMaxF; ++g) sp.grank[g] = p.grank[g];
    sp.rank_out = rank_out;
    sp.bucket_off = bucket_off;
    sp.bucket_idx = bucket_idx;
    const dim3 grid(split_layout(T, sp.per).G, B);
    hipLaunchKernelGGL(split_hist, grid, dim3(kSplitThreads), 0, stream, sp);
    hipLaunchKernelGGL(split_cand, grid, dim3(kSplitThreads), 0, stream, sp);
    hipLaunchKernelGGL(split_groups, grid, dim3(kSplitThreads), 0, stream, sp);
    hipLaunchKernelGGL(split_emit, grid, dim3(kSplitThreads), 0, stream, sp);
    p.split_ws = sp.ws;               // the one-workgroup kernel below: flagged rows only
    p.per = sp.per;
  }
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
