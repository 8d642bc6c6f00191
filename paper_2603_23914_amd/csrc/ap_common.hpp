// Shared host/device helpers of libattnpack (internal; not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>
#include "attnpack.h"

namespace ap {

// ---- error reporting (host) -------------------------------------------------
void set_error(const char* fmt, ...);
void clear_error();

#define AP_REQUIRE(cond, code, ...)        \
  do {                                     \
    if (!(cond)) {                         \
      ::ap::set_error(__VA_ARGS__);        \
      return (code);                       \
    }                                      \
  } while (0)

inline size_t dtype_size(ap_dtype dt) {
  switch (dt) {
    case AP_F32: return 4;
    case AP_F16: return 2;
    case AP_BF16: return 2;
    case AP_I8: return 1;
    case AP_I4: return 1;   // two coefficients per byte: callers that size rows use r / 2
  }
  return 0;
}
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- vector types used with the matrix-core builtins -------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2_t;

// ---- storage-type traits (device) --------------------------------------------
struct F16Tag {};
struct BF16Tag {};

// fp32 -> 16-bit storage, round to nearest even.
__device__ __forceinline__ uint16_t f32_to_bits(float x, F16Tag) {
  _Float16 h = (_Float16)x;  // v_cvt_f16_f32: RNE
  return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint16_t f32_to_bits(float x, BF16Tag) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bits_to_f32(uint16_t b, F16Tag) {
  return (float)__builtin_bit_cast(_Float16, b);
}
__device__ __forceinline__ float bits_to_f32(uint16_t b, BF16Tag) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}
// two packed 16-bit values in a dword (low half first in memory)
template <class Tag>
__device__ __forceinline__ float lo_to_f32(uint32_t w, Tag t) { return bits_to_f32((uint16_t)(w & 0xffffu), t); }
template <class Tag>
__device__ __forceinline__ float hi_to_f32(uint32_t w, Tag t) { return bits_to_f32((uint16_t)(w >> 16), t); }
template <class Tag>
__device__ __forceinline__ uint32_t pack2(float lo, float hi, Tag t) {
  return (uint32_t)f32_to_bits(lo, t) | ((uint32_t)f32_to_bits(hi, t) << 16);
}

// ---- launchers (defined in the .hip files) -------------------------------------
struct DecodeArgs {
  const void* q;
  const void* k_new;   // ap_decode_step only: [B, HD] rows appended at T-1 before attending
  const void* v_new;
  const void* Ck;
  const void* Cv;
  const void* scale_k;
  const void* scale_v;
  const void* Bk;
  const void* Bv;
  int64_t basis_batch_stride;
  const int32_t* rank_k;
  const int32_t* rank_v;
  const int32_t* bucket_off;
  const int32_t* bucket_idx;
  int F;
  void* out;
  float* lse;
  float* scores;       // [B, H, T_cap] scaled logits (natural-log units) of every attended token, or null
  int H_kv;            // key/value heads (grouped queries: H / H_kv query heads share one); bases are [r, H_kv*d]
  int B, H, d, T, T_cap, r;
  float sm_scale;
  ap_dtype dt, dt_coef, dt_out;
  void* workspace;
  size_t ws_bytes;
  hipStream_t stream;
};

size_t decode_f32_workspace(int B, int H, int d, int T, int r);
ap_status launch_decode_f32(const DecodeArgs& a);

size_t decode_mfma_workspace(int B, int H, int d, int T, int r, ap_dtype dt);
ap_status launch_decode_mfma(const DecodeArgs& a);

struct CompactArgs {
  const void* X;   // [B, n, HD]
  const void* Bm;  // [r, HD] (+ batch stride)
  void* C;         // [B, T_cap, r]
  void* scale;     // [B, T_cap, r/64] or null
  int B, n, row0, T_cap, HD, r;
  int64_t basis_batch_stride;
  ap_dtype dt_in, dt_out;
  hipStream_t stream;
};
ap_status launch_compact(const CompactArgs& a);
bool compact_gemm_applies(const CompactArgs& a);       // matrix-core path (compact_gemm.hip)
// General product of two 16-bit matrices that are contiguous along the contraction axis
// (compact_gemm.hip): C[b][m, j] = sum_k A[b][m, k] B[b][j, k].
struct NtGemmArgs {
  const void* A;  int64_t a_bstride; int lda;     // [M][K], elements
  const void* Bm; int64_t b_bstride; int ldb;     // [N][K] (b_bstride 0 = shared)
  void* C;        int64_t c_bstride; int ldc;     // [M][N] in elements of the output type
  void* scale;    int64_t s_bstride;              // out_kind 1: fp16 scales [M][N / 64]
  int batch, M, N, K;
  ap_dtype dt;                                    // AP_F16 or AP_BF16 (type of A and B)
  int out_kind;                                   // 0 = dt, 1 = int8 codes + scales, 2 = fp32
  hipStream_t stream;
};
ap_status launch_gemm_nt(const NtGemmArgs& a, const NtGemmArgs* second = nullptr);
// `second`: another projection of the same shape (B, n, row0, T_cap, HD, r, stride, types) that
// runs in the same launch, or null
ap_status launch_compact_gemm(const CompactArgs& a, const CompactArgs* second = nullptr);
ap_status launch_quantize_i8(const void* C, void* codes, void* scales, int B, int T, int T_cap,
                             int r, hipStream_t stream);
ap_status launch_quantize_i4(const void* C, void* codes, void* scales, int B, int T, int T_cap,
                             int r, hipStream_t stream);

// per-step passes over the bases in 16-bit storage (basis_gemv.hip)
bool basis_rows_applies(int HD, int B);
// ap_set_fused_value_min_bytes: -1 = the library's rule
int64_t fused_value_min_bytes();
ap_status launch_basis_rows(ap_dtype dt, const void* Bm, int64_t bstride, const void* x,
                            const void* q, void* C, void* Qp, int B, int H, int Hp, int d, int HD,
                            int r, int row0, int T_cap, float scale, hipStream_t stream,
                            const void* Bm2 = nullptr, const void* x2 = nullptr, void* C2 = nullptr);
int expand_row_blocks(int B, int r);   // row blocks (= partial output slices) of expand_append
ap_status launch_expand_append(ap_dtype dt, bool out_f32, const void* Bv, int64_t bstride,
                               const void* v_new, void* Cv, const float* part_ml,
                               const float* part_U, const float* pnew, const int* pnew_split,
                               const int32_t* rank_v, float* pout, void* out,
                               float* lse, int B, int H, int d, int r, int T, int T_cap, int nsplit,
                               hipStream_t stream);
ap_status launch_merge_splits(const float* part_ml, const float* part_U, float* out_ml, float* out_U,
                              float* pnew, const int* pnew_split, int B, int H, int r, int S,
                              hipStream_t stream);
ap_status launch_merge_expand(ap_dtype dt, bool out_f32, const float* part_ml, const float* part_U,
                              const void* Bv, int64_t bstride, void* out, float* lse, int B, int H,
                              int H_kv, int d, int r, int nsplit, hipStream_t stream);
ap_status launch_fold_heads(ap_dtype dt, const void* Bk, int64_t bstride, const void* q, void* Qp, int B,
                            int H, int H_kv, int Hp, int d, int r, float scale, hipStream_t stream);

ap_status launch_update_importance(const float* scores, const float* lse, float* mass, int B, int H,
                                   int T, int T_cap, int64_t mass_stride, float alpha,
                                   hipStream_t stream);

// measurement aid (probe.hip): plain streaming read
size_t probe_read_granule();
ap_status launch_probe_read(const void* src, size_t bytes, uint32_t* sink, bool non_temporal, hipStream_t stream);

size_t valueonly_attn_workspace(int B, int H, int H_kv, int d, int T, int r);
bool valueonly_rank_ok(int d, int r);
ap_status launch_valueonly_attn(const void* q, const void* K, const void* Cv, const void* Bv, int64_t bstride,
                                float* out, float* lse, int B, int H, int H_kv, int d, int T, int T_cap, int r,
                                float sm_scale, ap_dtype dt, void* workspace, hipStream_t stream);
// small uniform ranks (attn_small.hip): partial results in attn_partial's layout
bool attn_small_applies(int H, int r, int T, bool defer_v);
ap_status launch_attn_small(ap_dtype dt, const uint16_t* Qp, const void* Ck, const void* Cv, float* part_ml,
                            float* part_U, float* pnew, float* scores, const int32_t* rank_k,
                            const int32_t* rank_v, const int32_t* bucket_off, const int32_t* bucket_idx, int F,
                            int B, int H, int T, int T_cap, int r, int nsplit, bool defer_v,
                            hipStream_t stream);
// key-only compression on the matrix cores (keyonly_mfma.hip)
bool keyonly_mfma_applies(int H, int H_kv, int d, int r);
int keyonly_mfma_splits(int B, int H_kv, int T);
ap_status launch_keyonly_mfma(ap_dtype dt, const uint16_t* Qp, const void* Ck, const void* V, float* out_part,
                              float* lse_part, int B, int H, int H_kv, int T, int T_cap, int r, int S,
                              hipStream_t stream);
size_t keyonly_attn_workspace(int B, int H, int H_kv, int d, int T, int r);
ap_status launch_keyonly_attn(const void* q, const void* Ck, const void* Bk, int64_t bstride, const void* V,
                              float* out, float* lse, int B, int H, int H_kv, int d, int T, int T_cap, int r,
                              float sm_scale, ap_dtype dt, void* workspace, hipStream_t stream);
size_t raw_attn_workspace(int B, int H, int d, int T);
ap_status launch_raw_attn(const void* q, const void* K, const void* V, float* out, float* lse, int B,
                          int H, int H_kv, int d, int T, int T_cap, float sm_scale, ap_dtype dt,
                          void* workspace, hipStream_t stream);
ap_status launch_merge_segments(const float* out_a, const float* lse_a, const float* out_b,
                                const float* lse_b, void* out, float* lse, int B, int H, int d,
                                ap_dtype dt_out, hipStream_t stream);
ap_status launch_raw_append(const void* k_new, const void* v_new, void* K, void* V, int B, int HD, int row,
                            int T_cap, hipStream_t stream);

size_t select_workspace(int B, int T, int F);
ap_status launch_select_ranks(const float* mass, int B, int T, int F, const int32_t* group_rank,
                              const int32_t* bounds_num, int32_t den, int32_t* rank_out,
                              int32_t* bucket_off, int32_t* bucket_idx, void* ws,
                              hipStream_t stream);

// the compression step (bases.hip)
struct BasesArgs {
  const void* X;        // [B][n][HD]
  const void* Omega;    // [l][HD] start block (omega_batch_stride elements apart, 0 = shared)
  int64_t omega_batch_stride;
  void* Bm;             // out [B][r][HD]
  float* sigma;         // out [B][r] or null
  int B, n, HD, r, oversample, power_iters;
  ap_dtype dt;
  void* workspace;
  hipStream_t stream;
};
size_t bases_workspace(int B, int n, int HD, int r, int oversample);
ap_status launch_compute_bases(const BasesArgs& a);
size_t decompress_workspace(int B, int T, int HD, int r, bool ranks);
ap_status launch_decompress(const void* C, const void* Bm, int64_t bstride, const int32_t* rank, void* X, int B,
                            int T, int T_cap, int HD, int r, ap_dtype dt, void* workspace, hipStream_t stream);

ap_status check_launch(const char* what);

// dominant-kernel timing (api.hip): while timing is on, hands out the next pair of events; the
// caller attaches them to ONE kernel launch (hipExtLaunchKernelGGL), so their difference is
// that kernel's own start-to-end time, without the gap to the kernel before it
bool prof_events(hipEvent_t* start, hipEvent_t* stop);

}  // namespace ap
