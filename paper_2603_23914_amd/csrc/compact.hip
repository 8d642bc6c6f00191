// Compaction with given bases (paper Sec. 3.1: Kbar = K D_k^T) and the int8 coefficient
// format.
//
//   compact_rows : C[b, row0+i, j] = sum_c X[b, i, c] * Bm[b][j, c]      (fp32 accumulation)
//                  A workgroup owns RB rows x 64 columns.  The RB input rows stay in
//                  registers; each wave streams the basis rows of its 16 columns once with
//                  128-bit loads, so appending one token (n = 1, the per-step case) reads
//                  every basis byte exactly once: a bandwidth-bound matrix-vector product.
//                  Row blocks of 32 and more tokens in 16-bit types go to the matrix-core
//                  GEMM of compact_gemm.hip instead.
//   quantize     : per token and per 64 columns, amax -> fp16 scale -> int8 codes, in the
//                  exact fp32 / fp16 arithmetic the format prescribes.
#include "ap_common.hpp"

namespace ap {
namespace {

struct F32Tag {};
constexpr int kCols = 64;     // columns per workgroup (= one int8 scale block)

// 8 consecutive elements of a row, as loaded (kept packed in registers) and as floats
template <class Tag>
struct Pack {
  u32x4_t w;
  static constexpr int kBytes = 2;
  static constexpr int kPC = 10;      // 512-element passes of the hidden axis held in registers
  __device__ __forceinline__ void zero() { u32x4_t z = {0, 0, 0, 0}; w = z; }
  __device__ __forceinline__ void load(const void* p) { w = *(const u32x4_t*)p; }
  __device__ __forceinline__ void get(float (&v)[8]) const {
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[2 * e] = lo_to_f32(w[e], Tag{}); v[2 * e + 1] = hi_to_f32(w[e], Tag{}); }
  }
  static __device__ __forceinline__ void store(void* C, size_t idx, float v) {
    ((uint16_t*)C)[idx] = f32_to_bits(v, Tag{});
  }
};
template <>
struct Pack<F32Tag> {
  f32x4_t a, b;
  static constexpr int kBytes = 4;
  static constexpr int kPC = 4;
  __device__ __forceinline__ void zero() { f32x4_t z = {0.f, 0.f, 0.f, 0.f}; a = z; b = z; }
  __device__ __forceinline__ void load(const void* p) { a = *(const f32x4_t*)p; b = *((const f32x4_t*)p + 1); }
  __device__ __forceinline__ void get(float (&v)[8]) const {
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[e] = a[e]; v[4 + e] = b[e]; }
  }
  static __device__ __forceinline__ void store(void* C, size_t idx, float v) { ((float*)C)[idx] = v; }
};

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}

// One 64-column block of one token, one value per lane (already rounded to fp16):
// amax = max|c|;  scale = fp16(fp32(amax) / 127);  code = clamp(rint(fp32(c) / fp32(scale))).
__device__ __forceinline__ void quantize_block(float c, int8_t& code, uint16_t& scale_bits) {
  const float amax = wave_max(fabsf(c));
  const _Float16 sh = (_Float16)(amax / 127.0f);           // IEEE divide, RNE to fp16
  const float s = (float)sh;
  float q = 0.f;
  if (s != 0.f) q = fminf(fmaxf(rintf(c / s), -127.f), 127.f);
  code = (int8_t)(int)q;
  scale_bits = __builtin_bit_cast(uint16_t, sh);
}

template <class Tag, int RB>
__global__ void __launch_bounds__(256)
compact_rows(const void* __restrict__ X, const void* __restrict__ Bm, int64_t bstride,
             void* __restrict__ C, uint16_t* __restrict__ scale, int n, int row0, int T_cap,
             int HD, int r, int out_kind /* 0 = same type, 1 = int8 */) {
  constexpr int ES = Pack<Tag>::kBytes;
  constexpr int kPC = Pack<Tag>::kPC;
  __shared__ float tile[RB][kCols];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int j0 = blockIdx.x * kCols, i0 = blockIdx.y * RB, b = blockIdx.z;
  const char* Xb = (const char*)X + ((size_t)b * n + i0) * HD * ES;
  const char* Bb = (const char*)Bm + (size_t)b * bstride * ES;
  float acc[RB][16];
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int c = 0; c < 16; ++c) acc[i][c] = 0.f;

  for (int h0 = 0; h0 < HD; h0 += 512 * kPC) {
    // this lane's slice of the RB input rows for the chunk: elements h0 + 512*p + 8*lane ..
    Pack<Tag> x[RB][kPC];
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int p = 0; p < kPC; ++p) {
        const int h = h0 + 512 * p + 8 * lane;
        x[i][p].zero();
        if (h < HD && i0 + i < n) x[i][p].load(Xb + ((size_t)i * HD + h) * ES);
      }
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      const int j = j0 + 16 * w + c;
      if (j < r) {
        const char* brow = Bb + (size_t)j * HD * ES;
#pragma unroll
        for (int p = 0; p < kPC; ++p) {
          const int h = h0 + 512 * p + 8 * lane;
          if (h < HD) {
            Pack<Tag> bp;
            bp.load(brow + (size_t)h * ES);
            float bv[8];
            bp.get(bv);
#pragma unroll
            for (int i = 0; i < RB; ++i) {
              float xv[8];
              x[i][p].get(xv);
#pragma unroll
              for (int e = 0; e < 8; ++e) acc[i][c] = fmaf(xv[e], bv[e], acc[i][c]);
            }
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      const float s = wave_sum(acc[i][c]);
      if (lane == 0) tile[i][16 * w + c] = s;
    }
  __syncthreads();
  // epilogue: wave w finishes row i0 + w (+4, ...), one column per lane
  for (int i = w; i < RB; i += 4) {
    if (i0 + i >= n) break;
    const int j = j0 + lane;
    const size_t row = (size_t)b * T_cap + row0 + i0 + i;
    const float v = j < r ? tile[i][lane] : 0.f;
    if (out_kind == 1) {
      const float vh = (float)(_Float16)v;                  // the fp16 coefficient
      int8_t code;
      uint16_t sb;
      quantize_block(vh, code, sb);
      if (j < r) ((int8_t*)C)[row * r + j] = code;
      if (lane == 0) scale[row * (r / kCols) + blockIdx.x] = sb;
    } else if (j < r) {
      Pack<Tag>::store(C, row * r + j, v);
    }
  }
}

// grid (ceil(T / 4), B), 256 threads: a wave owns one token and walks its row 512 columns at a
// time (16-byte loads; 8 lanes share a 64-column scale block).
__global__ void __launch_bounds__(256)
quantize_i8(const uint16_t* __restrict__ C, int8_t* __restrict__ codes,
            uint16_t* __restrict__ scales, int T, int T_cap, int r) {
  const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6), b = blockIdx.y;
  if (t >= T) return;
  const size_t row = (size_t)b * T_cap + t;
  for (int c0 = 0; c0 < r; c0 += 512) {
    const int col = c0 + lane * 8;
    const bool live = col < r;
    u32x4_t v = {0, 0, 0, 0};
    if (live) v = *(const u32x4_t*)(C + row * r + col);
    float x[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) { x[2 * e] = lo_to_f32(v[e], F16Tag{}); x[2 * e + 1] = hi_to_f32(v[e], F16Tag{}); }
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(x[e]));
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    const _Float16 sh = (_Float16)(amax / 127.0f);          // IEEE divide, RNE to fp16
    const float s = (float)sh;
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float q = 0.f;
      if (s != 0.f) q = fminf(fmaxf(rintf(x[e] / s), -127.f), 127.f);
      const uint32_t byte = (uint32_t)(int)q & 0xffu;
      if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
    }
    if (live) {
      const u32x2_t cw = {lo, hi};
      *(u32x2_t*)(codes + row * r + col) = cw;
      if ((lane & 7) == 0) scales[row * (r / kCols) + (col >> 6)] = __builtin_bit_cast(uint16_t, sh);
    }
  }
}

// The 4-bit format: the same walk, codes -7 .. 7, two per byte (column 2i in the low nibble of
// byte i, each nibble the code plus 8).  A lane's 8 columns become one dword.
__global__ void __launch_bounds__(256)
quantize_i4(const uint16_t* __restrict__ C, uint8_t* __restrict__ codes,
            uint16_t* __restrict__ scales, int T, int T_cap, int r) {
  const int lane = threadIdx.x & 63, t = blockIdx.x * 4 + (threadIdx.x >> 6), b = blockIdx.y;
  if (t >= T) return;
  const size_t row = (size_t)b * T_cap + t;
  for (int c0 = 0; c0 < r; c0 += 512) {
    const int col = c0 + lane * 8;
    const bool live = col < r;
    u32x4_t v = {0, 0, 0, 0};
    if (live) v = *(const u32x4_t*)(C + row * r + col);
    float x[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) { x[2 * e] = lo_to_f32(v[e], F16Tag{}); x[2 * e + 1] = hi_to_f32(v[e], F16Tag{}); }
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(x[e]));
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    const _Float16 sh = (_Float16)(amax / 7.0f);             // IEEE divide, RNE to fp16
    const float s = (float)sh;
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float q = 0.f;
      if (s != 0.f) q = fminf(fmaxf(rintf(x[e] / s), -7.f), 7.f);
      word |= (uint32_t)((int)q + 8) << (4 * e);
    }
    if (live) {
      *(uint32_t*)(codes + row * (r >> 1) + (col >> 1)) = word;
      if ((lane & 7) == 0) scales[row * (r / kCols) + (col >> 6)] = __builtin_bit_cast(uint16_t, sh);
    }
  }
}

template <class Tag>
ap_status run_compact(const CompactArgs& a) {
  const int out_kind = a.dt_out == AP_I8 ? 1 : 0;
  const int jb = (a.r + kCols - 1) / kCols;
  if (a.n == 1) {
    hipLaunchKernelGGL((compact_rows<Tag, 1>), dim3(jb, 1, a.B), dim3(256), 0, a.stream, a.X, a.Bm,
                       a.basis_batch_stride, a.C, (uint16_t*)a.scale, a.n, a.row0, a.T_cap, a.HD,
                       a.r, out_kind);
  } else {
    hipLaunchKernelGGL((compact_rows<Tag, 4>), dim3(jb, (a.n + 3) / 4, a.B), dim3(256), 0, a.stream,
                       a.X, a.Bm, a.basis_batch_stride, a.C, (uint16_t*)a.scale, a.n, a.row0,
                       a.T_cap, a.HD, a.r, out_kind);
  }
  return check_launch("ap_compact");
}

}  // namespace

ap_status launch_compact(const CompactArgs& a) {
  if (compact_gemm_applies(a)) return launch_compact_gemm(a);
  if (a.n == 1 && a.dt_out == a.dt_in && (a.dt_in == AP_F16 || a.dt_in == AP_BF16) &&
      basis_rows_applies(a.HD, a.B)) {
    ap_status st = launch_basis_rows(a.dt_in, a.Bm, a.basis_batch_stride, a.X, nullptr, a.C, nullptr,
                                     a.B, 0, 0, 8, a.HD, a.r, a.row0, a.T_cap, 1.0f, a.stream);
    return st != AP_OK ? st : check_launch("ap_compact");
  }
  AP_REQUIRE(a.B <= 65535 && (a.n + 3) / 4 <= 65535, AP_ERR_UNSUPPORTED,
             "ap_compact: B and n/4 must be <= 65535");
  switch (a.dt_in) {
    case AP_F16: return run_compact<F16Tag>(a);
    case AP_BF16: return run_compact<BF16Tag>(a);
    case AP_F32: return run_compact<F32Tag>(a);
    default: break;
  }
  set_error("ap_compact: bad dt_in");
  return AP_ERR_INVALID_ARG;
}

ap_status launch_quantize_i8(const void* C, void* codes, void* scales, int B, int T, int T_cap,
                             int r, hipStream_t stream) {
  AP_REQUIRE(B <= 65535, AP_ERR_UNSUPPORTED, "ap_quantize_i8: B must be <= 65535");
  hipLaunchKernelGGL(quantize_i8, dim3((T + 3) / 4, B), dim3(256), 0, stream, (const uint16_t*)C,
                     (int8_t*)codes, (uint16_t*)scales, T, T_cap, r);
  return check_launch("ap_quantize_i8");
}

ap_status launch_quantize_i4(const void* C, void* codes, void* scales, int B, int T, int T_cap,
                             int r, hipStream_t stream) {
  AP_REQUIRE(B <= 65535, AP_ERR_UNSUPPORTED, "ap_quantize_i4: B must be <= 65535");
  hipLaunchKernelGGL(quantize_i4, dim3((T + 3) / 4, B), dim3(256), 0, stream, (const uint16_t*)C,
                     (uint8_t*)codes, (uint16_t*)scales, T, T_cap, r);
  return check_launch("ap_quantize_i4");
}

}  // namespace ap
