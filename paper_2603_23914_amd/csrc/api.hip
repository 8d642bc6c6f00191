// C ABI of libattnpack: host-side validation and dispatch.  No kernel lives here.
#include "ap_common.hpp"

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

// Scratch of ap_decode_attn_static: the decode workspace as a device array of the library itself.
// Every GPU that loads the library holds its own copy until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[AP_STATIC_SCRATCH_BYTES];

namespace ap {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap_;
  va_start(ap_, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap_);
  va_end(ap_);
}
void clear_error() { g_err[0] = 0; }

ap_status check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("%s: HIP error %d (%s)", what, (int)e, hipGetErrorString(e));
    return AP_ERR_HIP;
  }
  return AP_OK;
}

// ---- dominant-kernel timing ---------------------------------------------------------------
static bool g_prof_on = false;
static std::vector<hipEvent_t> g_prof_ev;   // start, stop, start, stop, ...
static size_t g_prof_used = 0;
static unsigned g_prof_every = 1, g_prof_seen = 0;
static int64_t g_fused_value_min_bytes = -1;
constexpr size_t kProfMax = 2 * 4096;

int64_t fused_value_min_bytes() { return g_fused_value_min_bytes; }

bool prof_events(hipEvent_t* start, hipEvent_t* stop) {
  if (!g_prof_on || g_prof_used + 2 > kProfMax) return false;
  if (g_prof_seen++ % g_prof_every != 0) return false;     // only every n-th launch carries events
  while (g_prof_ev.size() < g_prof_used + 2) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return false;
    g_prof_ev.push_back(e);
  }
  *start = g_prof_ev[g_prof_used];
  *stop = g_prof_ev[g_prof_used + 1];
  g_prof_used += 2;
  return true;
}

static bool half_type(ap_dtype dt) { return dt == AP_F16 || dt == AP_BF16; }

// Address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static ap_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("ap_decode_attn_static: no current device (%s)", e != hipSuccess ? hipGetErrorString(e) : "index out of range");
    return AP_ERR_HIP;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      set_error("ap_decode_attn_static: hipGetSymbolAddress failed (%s)", hipGetErrorString(e));
      return AP_ERR_HIP;
    }
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return AP_OK;
}

}  // namespace ap

using namespace ap;

extern "C" {

const char* ap_status_string(ap_status s) {
  switch (s) {
    case AP_OK: return "AP_OK";
    case AP_ERR_INVALID_ARG: return "AP_ERR_INVALID_ARG";
    case AP_ERR_UNSUPPORTED: return "AP_ERR_UNSUPPORTED";
    case AP_ERR_WORKSPACE: return "AP_ERR_WORKSPACE";
    case AP_ERR_HIP: return "AP_ERR_HIP";
  }
  return "AP_ERR_?";
}

const char* ap_last_error(void) { return g_err; }

int ap_version(void) { return 500; }   // 0.5.0: compression step, 4-bit coefficients, allocation-free decode entry

size_t ap_probe_read_granule(void) { return probe_read_granule(); }

ap_status ap_probe_read(const void* src, size_t bytes, void* sink, void* stream) {
  clear_error();
  AP_REQUIRE(src && sink, AP_ERR_INVALID_ARG, "ap_probe_read: NULL pointer");
  AP_REQUIRE(bytes > 0 && bytes % probe_read_granule() == 0, AP_ERR_INVALID_ARG,
             "ap_probe_read: bytes must be a positive multiple of %zu", probe_read_granule());
  AP_REQUIRE(aligned(src, 16) && aligned(sink, 4), AP_ERR_INVALID_ARG, "ap_probe_read: misaligned pointer");
  return launch_probe_read(src, bytes, (uint32_t*)sink, false, (hipStream_t)stream);
}

ap_status ap_probe_read_stream(const void* src, size_t bytes, void* sink, void* stream) {
  clear_error();
  AP_REQUIRE(src && sink, AP_ERR_INVALID_ARG, "ap_probe_read_stream: NULL pointer");
  AP_REQUIRE(bytes > 0 && bytes % probe_read_granule() == 0, AP_ERR_INVALID_ARG,
             "ap_probe_read_stream: bytes must be a positive multiple of %zu", probe_read_granule());
  AP_REQUIRE(aligned(src, 16) && aligned(sink, 4), AP_ERR_INVALID_ARG, "ap_probe_read_stream: misaligned pointer");
  return launch_probe_read(src, bytes, (uint32_t*)sink, true, (hipStream_t)stream);
}

void ap_set_fused_value_min_bytes(int64_t min_bytes) { g_fused_value_min_bytes = min_bytes < 0 ? -1 : min_bytes; }

void ap_prof_enable(int on) {
  g_prof_on = on > 0;
  g_prof_every = on > 0 ? (unsigned)on : 1u;
  g_prof_seen = 0;
  g_prof_used = 0;
}

ap_status ap_prof_read(float* total_ms, int* launches) {
  clear_error();
  AP_REQUIRE(total_ms && launches, AP_ERR_INVALID_ARG, "ap_prof_read: NULL pointer");
  const size_t pairs = g_prof_used / 2;
  float sum = 0.f;
  if (pairs) {
    hipError_t e = hipEventSynchronize(g_prof_ev[2 * pairs - 1]);
    if (e != hipSuccess) {
      set_error("ap_prof_read: %s", hipGetErrorString(e));
      return AP_ERR_HIP;
    }
    for (size_t i = 0; i < pairs; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, g_prof_ev[2 * i], g_prof_ev[2 * i + 1]) == hipSuccess) sum += ms;
    }
  }
  *total_ms = sum;
  *launches = (int)pairs;
  return AP_OK;
}

ap_status ap_prof_read_launches(float* us, int cap, int* launches) {
  clear_error();
  AP_REQUIRE(launches && (us || cap == 0) && cap >= 0, AP_ERR_INVALID_ARG, "ap_prof_read_launches: bad argument");
  const size_t pairs = g_prof_used / 2;
  if (pairs) {
    hipError_t e = hipEventSynchronize(g_prof_ev[2 * pairs - 1]);
    if (e != hipSuccess) {
      set_error("ap_prof_read_launches: %s", hipGetErrorString(e));
      return AP_ERR_HIP;
    }
    for (size_t i = 0; i < pairs && i < (size_t)cap; ++i) {
      float ms = 0.f;
      us[i] = hipEventElapsedTime(&ms, g_prof_ev[2 * i], g_prof_ev[2 * i + 1]) == hipSuccess ? ms * 1e3f : -1.f;
    }
  }
  *launches = (int)pairs;
  return AP_OK;
}

// ---------------------------------------------------------------------------------------------
ap_status ap_compact(const void* K, const void* V, const void* Bk, const void* Bv, void* Ck,
                     void* Cv, void* scale_k, void* scale_v, int B, int n, int row0, int T_cap,
                     int HD, int r, int64_t basis_batch_stride, ap_dtype dt_in, ap_dtype dt_out,
                     void* stream) {
  clear_error();
  AP_REQUIRE(B > 0 && n > 0 && HD > 0 && r > 0 && T_cap > 0, AP_ERR_INVALID_ARG,
             "ap_compact: B, n, T_cap, HD, r must be positive");
  AP_REQUIRE(row0 >= 0 && (int64_t)row0 + n <= T_cap, AP_ERR_INVALID_ARG,
             "ap_compact: rows [%d, %d) outside T_cap=%d", row0, row0 + n, T_cap);
  AP_REQUIRE(K != nullptr || V != nullptr, AP_ERR_INVALID_ARG, "ap_compact: K and V both NULL");
  AP_REQUIRE(dt_in == AP_F32 || half_type(dt_in), AP_ERR_INVALID_ARG, "ap_compact: bad dt_in");
  AP_REQUIRE(dt_out == dt_in || (dt_out == AP_I8 && dt_in == AP_F16), AP_ERR_INVALID_ARG,
             "ap_compact: dt_out must equal dt_in, or be AP_I8 with dt_in AP_F16");
  AP_REQUIRE(HD % 8 == 0 && r % 16 == 0, AP_ERR_INVALID_ARG,
             "ap_compact: need HD %% 8 == 0 and r %% 16 == 0 (HD=%d r=%d)", HD, r);
  AP_REQUIRE(basis_batch_stride == 0 || basis_batch_stride >= (int64_t)r * HD, AP_ERR_INVALID_ARG,
             "ap_compact: basis_batch_stride must be 0 or >= r*HD");
  AP_REQUIRE(basis_batch_stride % 8 == 0, AP_ERR_INVALID_ARG,
             "ap_compact: basis_batch_stride must keep rows 16-byte aligned");
  if (dt_out == AP_I8) {
    AP_REQUIRE(r % AP_QBLOCK == 0, AP_ERR_INVALID_ARG, "ap_compact: AP_I8 needs r %% 64 == 0");
  }
  const void* Xs[2] = {K, V};
  const void* Bs[2] = {Bk, Bv};
  void* Cs[2] = {Ck, Cv};
  void* Ss[2] = {scale_k, scale_v};
  for (int i = 0; i < 2; ++i) {
    if (!Xs[i]) continue;
    AP_REQUIRE(Bs[i] && Cs[i], AP_ERR_INVALID_ARG, "ap_compact: basis or output NULL for %s",
               i ? "V" : "K");
    AP_REQUIRE(aligned(Xs[i], 16) && aligned(Bs[i], 16) && aligned(Cs[i], 16), AP_ERR_INVALID_ARG,
               "ap_compact: %s pointers must be 16-byte aligned", i ? "V" : "K");
    if (dt_out == AP_I8)
      AP_REQUIRE(Ss[i] && aligned(Ss[i], 2), AP_ERR_INVALID_ARG,
                 "ap_compact: AP_I8 output needs a scale buffer");
  }
  if (Xs[0] && Xs[1]) {
    // keys and values of one prefill: both projections in one matrix-core launch when they qualify
    CompactArgs ak{Xs[0], Bs[0], Cs[0], Ss[0], B, n, row0, T_cap, HD, r, basis_batch_stride,
                   dt_in, dt_out, (hipStream_t)stream};
    CompactArgs av = ak;
    av.X = Xs[1]; av.Bm = Bs[1]; av.C = Cs[1]; av.scale = Ss[1];
    if (compact_gemm_applies(ak)) return launch_compact_gemm(ak, &av);
  }
  for (int i = 0; i < 2; ++i) {
    if (!Xs[i]) continue;
    CompactArgs a{Xs[i], Bs[i], Cs[i], Ss[i], B, n, row0, T_cap, HD, r, basis_batch_stride,
                  dt_in, dt_out, (hipStream_t)stream};
    ap_status s = launch_compact(a);
    if (s != AP_OK) return s;
  }
  return AP_OK;
}

// ---------------------------------------------------------------------------------------------
static bool bases_shape_ok(int B, int n, int HD, int r, int oversample) {
  const int64_t l = (int64_t)r + oversample;
  return B > 0 && B <= 65535 && n > 0 && HD > 0 && r > 0 && oversample >= 0 && HD % 64 == 0 && n % 8 == 0 &&
         l % 2 == 0 && l <= 1024 && l <= n && l <= HD;
}

size_t ap_bases_workspace_bytes(int B, int n, int HD, int r, int oversample) {
  return bases_shape_ok(B, n, HD, r, oversample) ? bases_workspace(B, n, HD, r, oversample) : 0;
}

ap_status ap_compute_bases(const void* X, const void* Omega, int64_t omega_batch_stride, void* Bm, float* sigma,
                           int B, int n, int HD, int r, int oversample, int power_iters, ap_dtype dt,
                           void* workspace, size_t ws_bytes, void* stream) {
  clear_error();
  AP_REQUIRE(X && Omega && Bm, AP_ERR_INVALID_ARG, "ap_compute_bases: NULL pointer");
  AP_REQUIRE(half_type(dt), AP_ERR_UNSUPPORTED, "ap_compute_bases: fp16 or bf16 storage only");
  AP_REQUIRE(B > 0 && n > 0 && HD > 0 && r > 0 && oversample >= 0 && power_iters >= 0 && power_iters <= 16,
             AP_ERR_INVALID_ARG, "ap_compute_bases: need B, n, HD, r > 0, oversample >= 0, 0 <= power_iters <= 16");
  AP_REQUIRE(bases_shape_ok(B, n, HD, r, oversample), AP_ERR_UNSUPPORTED,
             "ap_compute_bases: need HD %% 64 == 0, n %% 8 == 0, l = r + oversample even, l <= 1024, l <= n, "
             "l <= HD (n=%d HD=%d r=%d oversample=%d)", n, HD, r, oversample);
  const int64_t l = (int64_t)r + oversample;
  AP_REQUIRE(omega_batch_stride == 0 || omega_batch_stride >= l * HD, AP_ERR_INVALID_ARG,
             "ap_compute_bases: omega_batch_stride must be 0 or >= (r + oversample) * HD");
  AP_REQUIRE(aligned(X, 16) && aligned(Omega, 16) && aligned(Bm, 16) && aligned(workspace, 256), AP_ERR_INVALID_ARG,
             "ap_compute_bases: X, Omega, Bm must be 16-byte aligned, the workspace 256-byte");
  const size_t need = bases_workspace(B, n, HD, r, oversample);
  AP_REQUIRE(workspace && ws_bytes >= need, AP_ERR_WORKSPACE, "ap_compute_bases: workspace %zu bytes, need %zu",
             ws_bytes, need);
  BasesArgs a{X, Omega, omega_batch_stride, Bm, sigma, B, n, HD, r, oversample, power_iters, dt, workspace,
              (hipStream_t)stream};
  return launch_compute_bases(a);
}

size_t ap_decompress_workspace_bytes(int B, int T, int HD, int r, int with_ranks) {
  if (B <= 0 || T <= 0 || HD <= 0 || r <= 0) return 0;
  return decompress_workspace(B, T, HD, r, with_ranks != 0);
}

ap_status ap_decompress(const void* C, const void* Bm, int64_t basis_batch_stride, const int32_t* rank, void* X,
                        int B, int T, int T_cap, int HD, int r, ap_dtype dt, void* workspace, size_t ws_bytes,
                        void* stream) {
  clear_error();
  AP_REQUIRE(C && Bm && X, AP_ERR_INVALID_ARG, "ap_decompress: NULL pointer");
  AP_REQUIRE(half_type(dt), AP_ERR_UNSUPPORTED, "ap_decompress: fp16 or bf16 storage only");
  AP_REQUIRE(B > 0 && B <= 65535 && T > 0 && T <= T_cap && HD > 0 && r > 0, AP_ERR_INVALID_ARG,
             "ap_decompress: need 0 < B <= 65535, 0 < T <= T_cap, HD, r > 0");
  AP_REQUIRE(r % 64 == 0 && HD % 8 == 0, AP_ERR_UNSUPPORTED, "ap_decompress: need r %% 64 == 0 and HD %% 8 == 0");
  AP_REQUIRE(basis_batch_stride == 0 || basis_batch_stride >= (int64_t)r * HD, AP_ERR_INVALID_ARG,
             "ap_decompress: basis_batch_stride must be 0 or >= r*HD");
  AP_REQUIRE(aligned(C, 16) && aligned(Bm, 16) && aligned(X, 16) && aligned(workspace, 256), AP_ERR_INVALID_ARG,
             "ap_decompress: C, Bm, X must be 16-byte aligned, the workspace 256-byte");
  const size_t need = decompress_workspace(B, T, HD, r, rank != nullptr);
  AP_REQUIRE(workspace && ws_bytes >= need, AP_ERR_WORKSPACE, "ap_decompress: workspace %zu bytes, need %zu", ws_bytes,
             need);
  return launch_decompress(C, Bm, basis_batch_stride, rank, X, B, T, T_cap, HD, r, dt, workspace, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
ap_status ap_quantize_i8(const void* C, void* codes, void* scales, int B, int T, int T_cap, int r,
                         void* stream) {
  clear_error();
  AP_REQUIRE(C && codes && scales, AP_ERR_INVALID_ARG, "ap_quantize_i8: NULL pointer");
  AP_REQUIRE(B > 0 && T > 0 && T <= T_cap && r > 0, AP_ERR_INVALID_ARG,
             "ap_quantize_i8: need B > 0, 0 < T <= T_cap, r > 0");
  AP_REQUIRE(r % AP_QBLOCK == 0, AP_ERR_INVALID_ARG, "ap_quantize_i8: r %% 64 != 0");
  AP_REQUIRE(aligned(C, 16) && aligned(codes, 16) && aligned(scales, 2), AP_ERR_INVALID_ARG,
             "ap_quantize_i8: misaligned pointer");
  return launch_quantize_i8(C, codes, scales, B, T, T_cap, r, (hipStream_t)stream);
}

ap_status ap_quantize_i4(const void* C, void* codes, void* scales, int B, int T, int T_cap, int r,
                         void* stream) {
  clear_error();
  AP_REQUIRE(C && codes && scales, AP_ERR_INVALID_ARG, "ap_quantize_i4: NULL pointer");
  AP_REQUIRE(B > 0 && T > 0 && T <= T_cap && r > 0, AP_ERR_INVALID_ARG,
             "ap_quantize_i4: need B > 0, 0 < T <= T_cap, r > 0");
  AP_REQUIRE(r % AP_QBLOCK == 0, AP_ERR_INVALID_ARG, "ap_quantize_i4: r %% 64 != 0");
  AP_REQUIRE(aligned(C, 16) && aligned(codes, 16) && aligned(scales, 2), AP_ERR_INVALID_ARG,
             "ap_quantize_i4: misaligned pointer");
  return launch_quantize_i4(C, codes, scales, B, T, T_cap, r, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
size_t ap_select_workspace_bytes(int B, int T, int F) {
  if (B <= 0 || T <= 0 || F <= 0) return 0;
  return select_workspace(B, T, F);
}

ap_status ap_select_ranks(const float* mass, int B, int T, int F, const int32_t* group_rank,
                          const int32_t* cum_num, int32_t den, int32_t* rank_out,
                          int32_t* bucket_off, int32_t* bucket_idx, void* workspace,
                          size_t ws_bytes, void* stream) {
  clear_error();
  AP_REQUIRE(mass && group_rank && cum_num && rank_out && bucket_off && bucket_idx,
             AP_ERR_INVALID_ARG, "ap_select_ranks: NULL pointer");
  AP_REQUIRE(B > 0 && T > 0, AP_ERR_INVALID_ARG, "ap_select_ranks: B and T must be positive");
  AP_REQUIRE(F >= 1 && F <= 8, AP_ERR_INVALID_ARG, "ap_select_ranks: F must be in [1, 8]");
  AP_REQUIRE(den > 0, AP_ERR_INVALID_ARG, "ap_select_ranks: den must be positive");
  for (int g = 0; g < F; ++g) {
    AP_REQUIRE(group_rank[g] > 0, AP_ERR_INVALID_ARG, "ap_select_ranks: group_rank[%d] <= 0", g);
    AP_REQUIRE(g == 0 || group_rank[g] <= group_rank[g - 1], AP_ERR_INVALID_ARG,
               "ap_select_ranks: group_rank must be non-increasing");
    AP_REQUIRE(cum_num[g] >= (g ? cum_num[g - 1] : 0) && cum_num[g] <= den, AP_ERR_INVALID_ARG,
               "ap_select_ranks: cum_num must be non-decreasing within [0, den]");
  }
  AP_REQUIRE(cum_num[F - 1] == den, AP_ERR_INVALID_ARG, "ap_select_ranks: cum_num[F-1] != den");
  size_t need = select_workspace(B, T, F);
  AP_REQUIRE(workspace && ws_bytes >= need, AP_ERR_WORKSPACE,
             "ap_select_ranks: workspace %zu bytes, need %zu", ws_bytes, need);
  AP_REQUIRE(aligned(workspace, 16), AP_ERR_INVALID_ARG, "ap_select_ranks: workspace misaligned");
  return launch_select_ranks(mass, B, T, F, group_rank, cum_num, den, rank_out, bucket_off,
                             bucket_idx, workspace, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
static ap_status decode_shape_check(int B, int H, int d, int T, int r, ap_dtype dt, bool report) {
  if (B <= 0 || H <= 0 || d <= 0 || T <= 0 || r <= 0) {
    if (report) set_error("ap_decode_attn: B, H, d, T, r must be positive");
    return AP_ERR_INVALID_ARG;
  }
  if (dt == AP_F32) return AP_OK;
  if (!half_type(dt)) {
    if (report) set_error("ap_decode_attn: dt must be AP_F32, AP_F16 or AP_BF16");
    return AP_ERR_INVALID_ARG;
  }
  bool ok = H <= 64 && (d == 32 || d == 64 || d == 128 || d == 256) && r % 64 == 0 && r <= 640;
  if (!ok) {
    if (report)
      set_error("ap_decode_attn: half-precision path needs H<=64, d in {32,64,128,256}, "
                "r%%64==0, r<=640 (H=%d d=%d r=%d)", H, d, r);
    return AP_ERR_UNSUPPORTED;
  }
  return AP_OK;
}

size_t ap_decode_workspace_bytes(int B, int H, int d, int T, int r, ap_dtype dt) {
  if (decode_shape_check(B, H, d, T, r, dt, false) != AP_OK) return 0;
  return dt == AP_F32 ? decode_f32_workspace(B, H, d, T, r)
                      : decode_mfma_workspace(B, H, d, T, r, dt);
}

static ap_status decode_entry(const char* name, const void* q, const void* k_new, const void* v_new,
                              const void* Ck, const void* Cv, const void* scale_k,
                              const void* scale_v, const void* Bk, const void* Bv,
                              int64_t basis_batch_stride, const int32_t* rank_k,
                              const int32_t* rank_v, const int32_t* bucket_off,
                              const int32_t* bucket_idx, int F, void* out, float* lse, float* scores,
                              int B, int H, int H_kv, int d, int T, int T_cap, int r, float sm_scale,
                              ap_dtype dt,
                              ap_dtype dt_coef, ap_dtype dt_out, void* workspace, size_t ws_bytes,
                              void* stream) {
  clear_error();
  AP_REQUIRE(q && Ck && Cv && Bk && Bv && out, AP_ERR_INVALID_ARG, "%s: NULL pointer", name);
  ap_status s = decode_shape_check(B, H, d, T, r, dt, true);
  if (s != AP_OK) return s;
  AP_REQUIRE(T <= T_cap, AP_ERR_INVALID_ARG, "%s: T=%d exceeds T_cap=%d", name, T, T_cap);
  AP_REQUIRE(dt_coef == dt || ((dt_coef == AP_I8 || dt_coef == AP_I4) && dt == AP_F16), AP_ERR_INVALID_ARG,
             "%s: dt_coef must equal dt, or be AP_I8 / AP_I4 with dt AP_F16", name);
  AP_REQUIRE(dt_out == dt || dt_out == AP_F32, AP_ERR_INVALID_ARG,
             "%s: dt_out must equal dt or be AP_F32", name);
  AP_REQUIRE(sm_scale == sm_scale && sm_scale > 0.f && sm_scale < 1e30f, AP_ERR_INVALID_ARG,
             "%s: sm_scale must be finite and positive", name);
  AP_REQUIRE(H_kv >= 1 && H % H_kv == 0, AP_ERR_INVALID_ARG,
             "%s: H_kv=%d must be positive and divide H=%d", name, H_kv, H);
  const int64_t HD = (int64_t)H_kv * d;
  AP_REQUIRE(basis_batch_stride == 0 || basis_batch_stride >= (int64_t)r * HD, AP_ERR_INVALID_ARG,
             "%s: basis_batch_stride must be 0 or >= r*H_kv*d", name);
  AP_REQUIRE(aligned(q, 16) && aligned(Ck, 16) && aligned(Cv, 16) && aligned(Bk, 16) &&
                 aligned(Bv, 16) && aligned(out, 16),
             AP_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", name);
  AP_REQUIRE(aligned(scores, 16), AP_ERR_INVALID_ARG, "%s: scores must be 16-byte aligned", name);
  if (dt != AP_F32) {
    AP_REQUIRE(basis_batch_stride % 8 == 0, AP_ERR_INVALID_ARG,
               "%s: basis_batch_stride must keep rows 16-byte aligned", name);
  }
  if (dt_coef == AP_I8 || dt_coef == AP_I4) {
    AP_REQUIRE(scale_k && scale_v, AP_ERR_INVALID_ARG, "%s: quantised coefficients need scale buffers", name);
  }
  if (k_new || v_new) {
    AP_REQUIRE(k_new && v_new && aligned(k_new, 16) && aligned(v_new, 16), AP_ERR_INVALID_ARG,
               "%s: k_new and v_new must both be given, 16-byte aligned", name);
    AP_REQUIRE(half_type(dt) && dt_coef == dt, AP_ERR_UNSUPPORTED,
               "%s: the fused append needs AP_F16 / AP_BF16 coefficients of the same type", name);
  }
  const bool ragged = rank_k || rank_v;
  if (ragged && dt != AP_F32) {
    AP_REQUIRE(bucket_off && bucket_idx && F >= 1 && F <= 8, AP_ERR_INVALID_ARG,
               "%s: per-token ranks need the bucket lists of ap_select_ranks "
               "(1 <= F <= 8) in half precision", name);
  }
  size_t need = ap_decode_workspace_bytes(B, H, d, T, r, dt);
  AP_REQUIRE(workspace && ws_bytes >= need, AP_ERR_WORKSPACE, "%s: workspace %zu bytes, need %zu",
             name, ws_bytes, need);
  AP_REQUIRE(aligned(workspace, 256), AP_ERR_INVALID_ARG, "%s: workspace must be 256-byte aligned",
             name);
  DecodeArgs a{q, k_new, v_new, Ck, Cv, scale_k, scale_v, Bk, Bv, basis_batch_stride, rank_k, rank_v,
               bucket_off, bucket_idx, ragged ? F : 0, out, lse, scores, H_kv, B, H, d, T, T_cap, r, sm_scale,
               dt, dt_coef, dt_out, workspace, ws_bytes, (hipStream_t)stream};
  return dt == AP_F32 ? launch_decode_f32(a) : launch_decode_mfma(a);
}

ap_status ap_decode_attn(const void* q, const void* Ck, const void* Cv, const void* scale_k,
                         const void* scale_v, const void* Bk, const void* Bv,
                         int64_t basis_batch_stride, const int32_t* rank_k, const int32_t* rank_v,
                         const int32_t* bucket_off, const int32_t* bucket_idx, int F, void* out,
                         float* lse, float* scores, int B, int H, int H_kv, int d, int T, int T_cap,
                         int r, float sm_scale, ap_dtype dt, ap_dtype dt_coef, ap_dtype dt_out,
                         void* workspace, size_t ws_bytes, void* stream) {
  return decode_entry("ap_decode_attn", q, nullptr, nullptr, Ck, Cv, scale_k, scale_v, Bk, Bv,
                      basis_batch_stride, rank_k, rank_v, bucket_off, bucket_idx, F, out, lse, scores, B, H, H_kv,
                      d, T, T_cap, r, sm_scale, dt, dt_coef, dt_out, workspace, ws_bytes, stream);
}

ap_status ap_decode_attn_static(const void* q, const void* Ck, const void* Cv, const void* scale_k,
                                const void* scale_v, const void* Bk, const void* Bv,
                                int64_t basis_batch_stride, const int32_t* rank_k,
                                const int32_t* rank_v, const int32_t* bucket_off,
                                const int32_t* bucket_idx, int F, void* out, float* lse, float* scores,
                                int B, int H, int H_kv, int d, int T, int T_cap, int r, float sm_scale,
                                ap_dtype dt, ap_dtype dt_coef, ap_dtype dt_out, void* stream) {
  clear_error();
  ap_status s = decode_shape_check(B, H, d, T, r, dt, true);
  if (s != AP_OK) return s;
  const size_t need = ap_decode_workspace_bytes(B, H, d, T, r, dt);
  AP_REQUIRE(need <= (size_t)AP_STATIC_SCRATCH_BYTES, AP_ERR_WORKSPACE,
             "ap_decode_attn_static: this shape needs %zu bytes of scratch, the library's buffer holds %zu "
             "(use ap_decode_attn with a workspace of the caller)", need, (size_t)AP_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  s = static_scratch(&ws);
  if (s != AP_OK) return s;
  return decode_entry("ap_decode_attn_static", q, nullptr, nullptr, Ck, Cv, scale_k, scale_v, Bk, Bv,
                      basis_batch_stride, rank_k, rank_v, bucket_off, bucket_idx, F, out, lse, scores, B, H,
                      H_kv, d, T, T_cap, r, sm_scale, dt, dt_coef, dt_out, ws, (size_t)AP_STATIC_SCRATCH_BYTES,
                      stream);
}

ap_status ap_decode_step(const void* q, const void* k_new, const void* v_new, void* Ck, void* Cv,
                         const void* Bk, const void* Bv, int64_t basis_batch_stride,
                         const int32_t* rank_k, const int32_t* rank_v, const int32_t* bucket_off,
                         const int32_t* bucket_idx, int F, void* out, float* lse, float* scores,
                         int B, int H, int H_kv, int d, int T, int T_cap, int r, float sm_scale,
                         ap_dtype dt, ap_dtype dt_out, void* workspace, size_t ws_bytes, void* stream) {
  clear_error();
  AP_REQUIRE(k_new && v_new, AP_ERR_INVALID_ARG, "ap_decode_step: NULL pointer");
  return decode_entry("ap_decode_step", q, k_new, v_new, Ck, Cv, nullptr, nullptr, Bk, Bv,
                      basis_batch_stride, rank_k, rank_v, bucket_off, bucket_idx, F, out, lse, scores, B, H, H_kv,
                      d, T, T_cap, r, sm_scale, dt, dt, dt_out, workspace, ws_bytes, stream);
}

static bool raw_shape_ok(int B, int H, int d) {
  return B > 0 && B <= 65535 && H > 0 && H <= 65535 && (d == 32 || d == 64 || d == 128 || d == 256);
}

size_t ap_raw_workspace_bytes(int B, int H, int d, int T_u) {
  if (!raw_shape_ok(B, H, d) || T_u < 0) return 0;
  return raw_attn_workspace(B, H, d, T_u);
}

ap_status ap_raw_attn(const void* q, const void* K, const void* V, float* out, float* lse, int B, int H,
                      int H_kv, int d, int T_u, int T_u_cap, float sm_scale, ap_dtype dt, void* workspace,
                      size_t ws_bytes, void* stream) {
  clear_error();
  AP_REQUIRE(q && out && workspace, AP_ERR_INVALID_ARG, "ap_raw_attn: NULL pointer");
  AP_REQUIRE(raw_shape_ok(B, H, d), AP_ERR_UNSUPPORTED,
             "ap_raw_attn: need 0 < B, H <= 65535 and d in {32, 64, 128, 256}");
  AP_REQUIRE(H_kv >= 1 && H % H_kv == 0, AP_ERR_INVALID_ARG,
             "ap_raw_attn: H_kv=%d must be positive and divide H=%d", H_kv, H);
  AP_REQUIRE(dt == AP_F16 || dt == AP_BF16, AP_ERR_UNSUPPORTED, "ap_raw_attn: fp16 or bf16 storage only");
  AP_REQUIRE(T_u >= 0 && T_u <= T_u_cap, AP_ERR_INVALID_ARG, "ap_raw_attn: need 0 <= T_u <= T_u_cap");
  AP_REQUIRE(T_u == 0 || (K && V), AP_ERR_INVALID_ARG, "ap_raw_attn: NULL cache with T_u > 0");
  AP_REQUIRE(aligned(q, 16) && aligned(K, 16) && aligned(V, 16), AP_ERR_INVALID_ARG,
             "ap_raw_attn: q, K, V must be 16-byte aligned");
  AP_REQUIRE(ws_bytes >= raw_attn_workspace(B, H, d, T_u), AP_ERR_WORKSPACE,
             "ap_raw_attn: workspace too small (%zu < %zu bytes)", ws_bytes,
             raw_attn_workspace(B, H, d, T_u));
  return launch_raw_attn(q, K, V, out, lse, B, H, H_kv, d, T_u, T_u_cap, sm_scale, dt, workspace,
                         (hipStream_t)stream);
}

size_t ap_keyonly_workspace_bytes(int B, int H, int H_kv, int d, int T, int r) {
  if (!raw_shape_ok(B, H, d) || T < 0 || r <= 0 || r > 640 || r % 8 != 0) return 0;
  if (H_kv < 1 || H % H_kv != 0) return 0;
  return keyonly_attn_workspace(B, H, H_kv, d, T, r);
}

ap_status ap_keyonly_attn(const void* q, const void* Ck, const void* Bk, int64_t basis_batch_stride,
                          const void* V, float* out, float* lse, int B, int H, int H_kv, int d, int T,
                          int T_cap, int r, float sm_scale, ap_dtype dt, void* workspace, size_t ws_bytes,
                          void* stream) {
  clear_error();
  AP_REQUIRE(q && Bk && out && workspace, AP_ERR_INVALID_ARG, "ap_keyonly_attn: NULL pointer");
  AP_REQUIRE(raw_shape_ok(B, H, d), AP_ERR_UNSUPPORTED,
             "ap_keyonly_attn: need 0 < B, H <= 65535 and d in {32, 64, 128, 256}");
  AP_REQUIRE(H_kv >= 1 && H % H_kv == 0, AP_ERR_INVALID_ARG,
             "ap_keyonly_attn: H_kv=%d must be positive and divide H=%d", H_kv, H);
  AP_REQUIRE(dt == AP_F16 || dt == AP_BF16, AP_ERR_UNSUPPORTED, "ap_keyonly_attn: fp16 or bf16 storage only");
  AP_REQUIRE(r > 0 && r % 8 == 0, AP_ERR_INVALID_ARG, "ap_keyonly_attn: r=%d must be a positive multiple of 8", r);
  AP_REQUIRE(r <= 640, AP_ERR_UNSUPPORTED, "ap_keyonly_attn: r=%d exceeds 640", r);
  AP_REQUIRE(T >= 0 && T <= T_cap, AP_ERR_INVALID_ARG, "ap_keyonly_attn: need 0 <= T <= T_cap");
  AP_REQUIRE(T == 0 || (Ck && V), AP_ERR_INVALID_ARG, "ap_keyonly_attn: NULL cache with T > 0");
  const int64_t HDkv = (int64_t)H_kv * d;
  AP_REQUIRE(basis_batch_stride == 0 || basis_batch_stride >= (int64_t)r * HDkv, AP_ERR_INVALID_ARG,
             "ap_keyonly_attn: basis_batch_stride must be 0 or >= r*H_kv*d");
  AP_REQUIRE(basis_batch_stride % 8 == 0, AP_ERR_INVALID_ARG,
             "ap_keyonly_attn: basis_batch_stride must keep rows 16-byte aligned");
  AP_REQUIRE(aligned(q, 16) && aligned(Ck, 16) && aligned(Bk, 16) && aligned(V, 16) && aligned(workspace, 256),
             AP_ERR_INVALID_ARG, "ap_keyonly_attn: q, Ck, Bk, V must be 16-byte aligned, the workspace 256-byte");
  AP_REQUIRE(ws_bytes >= keyonly_attn_workspace(B, H, H_kv, d, T, r), AP_ERR_WORKSPACE,
             "ap_keyonly_attn: workspace too small (%zu < %zu bytes)", ws_bytes,
             keyonly_attn_workspace(B, H, H_kv, d, T, r));
  return launch_keyonly_attn(q, Ck, Bk, basis_batch_stride, V, out, lse, B, H, H_kv, d, T, T_cap, r, sm_scale,
                             dt, workspace, (hipStream_t)stream);
}

size_t ap_valueonly_workspace_bytes(int B, int H, int H_kv, int d, int T, int r) {
  if (!raw_shape_ok(B, H, d) || T < 1 || r <= 0 || r % 8 != 0 || !valueonly_rank_ok(d, r)) return 0;
  if (H_kv < 1 || H % H_kv != 0) return 0;
  return valueonly_attn_workspace(B, H, H_kv, d, T, r);
}

ap_status ap_valueonly_attn(const void* q, const void* K, const void* Cv, const void* Bv,
                            int64_t basis_batch_stride, float* out, float* lse, int B, int H, int H_kv,
                            int d, int T, int T_cap, int r, float sm_scale, ap_dtype dt, void* workspace,
                            size_t ws_bytes, void* stream) {
  clear_error();
  AP_REQUIRE(q && K && Cv && Bv && out && workspace, AP_ERR_INVALID_ARG, "ap_valueonly_attn: NULL pointer");
  AP_REQUIRE(raw_shape_ok(B, H, d), AP_ERR_UNSUPPORTED,
             "ap_valueonly_attn: need 0 < B, H <= 65535 and d in {32, 64, 128, 256}");
  AP_REQUIRE(H_kv >= 1 && H % H_kv == 0, AP_ERR_INVALID_ARG,
             "ap_valueonly_attn: H_kv=%d must be positive and divide H=%d", H_kv, H);
  AP_REQUIRE(dt == AP_F16 || dt == AP_BF16, AP_ERR_UNSUPPORTED, "ap_valueonly_attn: fp16 or bf16 storage only");
  AP_REQUIRE(r > 0 && r % 8 == 0, AP_ERR_INVALID_ARG, "ap_valueonly_attn: r=%d must be a positive multiple of 8", r);
  AP_REQUIRE(valueonly_rank_ok(d, r), AP_ERR_UNSUPPORTED,
             "ap_valueonly_attn: r=%d exceeds the limit for d=%d (640; 320 at d=32)", r, d);
  AP_REQUIRE(T >= 1 && T <= T_cap, AP_ERR_INVALID_ARG, "ap_valueonly_attn: need 1 <= T <= T_cap");
  const int64_t HDkv = (int64_t)H_kv * d;
  AP_REQUIRE(HDkv <= 8192, AP_ERR_UNSUPPORTED, "ap_valueonly_attn: H_kv*d must be <= 8192");
  AP_REQUIRE(basis_batch_stride == 0 || basis_batch_stride >= (int64_t)r * HDkv, AP_ERR_INVALID_ARG,
             "ap_valueonly_attn: basis_batch_stride must be 0 or >= r*H_kv*d");
  AP_REQUIRE(basis_batch_stride % 8 == 0, AP_ERR_INVALID_ARG,
             "ap_valueonly_attn: basis_batch_stride must keep rows 16-byte aligned");
  AP_REQUIRE(aligned(q, 16) && aligned(K, 16) && aligned(Cv, 16) && aligned(Bv, 16) && aligned(workspace, 256),
             AP_ERR_INVALID_ARG, "ap_valueonly_attn: q, K, Cv, Bv must be 16-byte aligned, the workspace 256-byte");
  AP_REQUIRE(ws_bytes >= valueonly_attn_workspace(B, H, H_kv, d, T, r), AP_ERR_WORKSPACE,
             "ap_valueonly_attn: workspace too small (%zu < %zu bytes)", ws_bytes,
             valueonly_attn_workspace(B, H, H_kv, d, T, r));
  return launch_valueonly_attn(q, K, Cv, Bv, basis_batch_stride, out, lse, B, H, H_kv, d, T, T_cap, r, sm_scale,
                               dt, workspace, (hipStream_t)stream);
}

ap_status ap_merge_segments(const float* out_a, const float* lse_a, const float* out_b,
                            const float* lse_b, void* out, float* lse, int B, int H, int d,
                            ap_dtype dt_out, void* stream) {
  clear_error();
  AP_REQUIRE(out_a && lse_a && out_b && lse_b && out, AP_ERR_INVALID_ARG, "ap_merge_segments: NULL pointer");
  AP_REQUIRE(B > 0 && B <= 65535 && H > 0 && d > 0, AP_ERR_INVALID_ARG,
             "ap_merge_segments: need 0 < B <= 65535, H > 0, d > 0");
  AP_REQUIRE(dt_out == AP_F32 || dt_out == AP_F16 || dt_out == AP_BF16, AP_ERR_UNSUPPORTED,
             "ap_merge_segments: output type must be fp32, fp16 or bf16");
  return launch_merge_segments(out_a, lse_a, out_b, lse_b, out, lse, B, H, d, dt_out, (hipStream_t)stream);
}

ap_status ap_raw_append(const void* k_new, const void* v_new, void* K, void* V, int B, int HD, int row,
                        int T_u_cap, ap_dtype dt, void* stream) {
  clear_error();
  AP_REQUIRE((k_new && K) || (v_new && V), AP_ERR_INVALID_ARG, "ap_raw_append: nothing to append");
  AP_REQUIRE((!k_new || K) && (!v_new || V), AP_ERR_INVALID_ARG, "ap_raw_append: row without its cache");
  AP_REQUIRE(dt == AP_F16 || dt == AP_BF16, AP_ERR_UNSUPPORTED, "ap_raw_append: fp16 or bf16 storage only");
  AP_REQUIRE(B > 0 && B <= 65535 && HD > 0 && HD % 8 == 0, AP_ERR_INVALID_ARG,
             "ap_raw_append: need 0 < B <= 65535 and HD a positive multiple of 8");
  AP_REQUIRE(row >= 0 && row < T_u_cap, AP_ERR_INVALID_ARG, "ap_raw_append: need 0 <= row < T_u_cap");
  AP_REQUIRE(aligned(k_new, 16) && aligned(v_new, 16) && aligned(K, 16) && aligned(V, 16),
             AP_ERR_INVALID_ARG, "ap_raw_append: pointers must be 16-byte aligned");
  return launch_raw_append(k_new, v_new, K, V, B, HD, row, T_u_cap, (hipStream_t)stream);
}

ap_status ap_update_importance(const float* scores, const float* lse, float* mass, int B, int H,
                               int T, int T_cap, int64_t mass_stride, float alpha, void* stream) {
  clear_error();
  AP_REQUIRE(scores && lse && mass, AP_ERR_INVALID_ARG, "ap_update_importance: NULL pointer");
  AP_REQUIRE(B > 0 && H > 0 && T > 0 && T <= T_cap && mass_stride >= T, AP_ERR_INVALID_ARG,
             "ap_update_importance: need B, H > 0, 0 < T <= T_cap, mass_stride >= T");
  AP_REQUIRE(alpha >= 0.f && alpha <= 1.f, AP_ERR_INVALID_ARG,
             "ap_update_importance: alpha must lie in [0, 1]");
  AP_REQUIRE(B <= 65535, AP_ERR_UNSUPPORTED, "ap_update_importance: B must be <= 65535");
  return launch_update_importance(scores, lse, mass, B, H, T, T_cap, mass_stride, alpha,
                                  (hipStream_t)stream);
}

}  // extern "C"
