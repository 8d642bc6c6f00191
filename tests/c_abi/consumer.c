/* A plain C99 consumer of the attnpack C ABI: no C++, no Python and no torch in the process.
 *
 *   consumer host                 host-only entry points and argument validation (needs no GPU)
 *   consumer run IN.bin OUT.bin   one ap_decode_attn or ap_decode_step call on the case in IN.bin
 *
 * IN.bin:  int32 header[12] = {magic, B, H, H_kv, d, T, T_cap, r, dt, step, shared_basis, bits of
 *          sm_scale}, then q [B,H,d], (k_new, v_new [B,H_kv*d] when step), Ck, Cv [B,T_cap,r],
 *          Bk, Bv [r,H_kv*d] (shared) or [B,r,H_kv*d], all in the storage type dt.
 * OUT.bin: out [B,H,d] fp32, lse [B,H] fp32, then (when step) row T-1 of Ck and of Cv [B,r] in dt.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "attnpack.h"

#define MAGIC 0x41504b31 /* "APK1" */

#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) {                                                          \
      fprintf(stderr, "consumer: line %d: %s is false (last error: %s)\n", __LINE__, #cond, ap_last_error()); \
      return 1;                                                             \
    }                                                                       \
  } while (0)

#define HIP_OK(call)                                                        \
  do {                                                                      \
    hipError_t e_ = (call);                                                 \
    if (e_ != hipSuccess) {                                                 \
      fprintf(stderr, "consumer: %s: %s\n", #call, hipGetErrorString(e_));  \
      return 2;                                                             \
    }                                                                       \
  } while (0)

static int host_checks(void) {
  EXPECT(ap_version() >= 400);
  EXPECT(strcmp(ap_status_string(AP_OK), "AP_OK") == 0);
  EXPECT(strcmp(ap_status_string(AP_ERR_WORKSPACE), "AP_ERR_WORKSPACE") == 0);
  EXPECT(ap_decode_workspace_bytes(64, 40, 128, 4288, 640, AP_BF16) > 0);
  EXPECT(ap_decode_workspace_bytes(0, 40, 128, 4288, 640, AP_BF16) == 0);
  EXPECT(ap_select_workspace_bytes(1, 32768, 4) > 0);
  EXPECT(ap_raw_workspace_bytes(8, 32, 128, 8192) > 0);
  EXPECT(ap_keyonly_workspace_bytes(8, 32, 8, 128, 8192, 64) > 0);
  EXPECT(ap_keyonly_workspace_bytes(8, 32, 5, 128, 8192, 64) == 0);
  EXPECT(ap_valueonly_workspace_bytes(8, 32, 8, 128, 8192, 256) > 0);
  EXPECT(ap_probe_read_granule() % 16 == 0);
  /* NULL pointers are refused before anything is launched */
  EXPECT(ap_decode_attn(NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL, NULL, NULL, NULL, 0, NULL, NULL, NULL,
                        1, 4, 4, 32, 64, 64, 16, 0.1f, AP_F32, AP_F32, AP_F32, NULL, 0, NULL) == AP_ERR_INVALID_ARG);
  EXPECT(strstr(ap_last_error(), "NULL") != NULL);
  EXPECT(ap_raw_attn(NULL, NULL, NULL, NULL, NULL, 1, 4, 4, 32, 8, 8, 0.1f, AP_F16, NULL, 0, NULL) ==
         AP_ERR_INVALID_ARG);
  EXPECT(ap_keyonly_attn(NULL, NULL, NULL, 0, NULL, NULL, NULL, 1, 4, 4, 32, 8, 8, 16, 0.1f, AP_F16, NULL, 0, NULL) ==
         AP_ERR_INVALID_ARG);
  EXPECT(ap_merge_segments(NULL, NULL, NULL, NULL, NULL, NULL, 1, 4, 32, AP_F32, NULL) == AP_ERR_INVALID_ARG);
  printf("consumer: host checks passed (library version %d)\n", ap_version());
  return 0;
}

static size_t elt_bytes(int dt) { return dt == AP_F32 ? 4 : 2; }

static int run_case(const char* in_path, const char* out_path) {
  FILE* f = fopen(in_path, "rb");
  if (!f) { perror(in_path); return 2; }
  int32_t hd[12];
  if (fread(hd, sizeof hd, 1, f) != 1 || hd[0] != MAGIC) { fprintf(stderr, "consumer: bad header\n"); return 2; }
  const int B = hd[1], H = hd[2], Hkv = hd[3], d = hd[4], T = hd[5], T_cap = hd[6], r = hd[7], dt = hd[8];
  const int step = hd[9], shared = hd[10];
  float sm_scale;
  memcpy(&sm_scale, &hd[11], 4);
  const size_t es = elt_bytes(dt), HD = (size_t)Hkv * d;
  const size_t n_q = (size_t)B * H * d, n_new = (size_t)B * HD, n_c = (size_t)B * T_cap * r;
  const size_t n_b = (shared ? 1 : (size_t)B) * r * HD;
  const size_t sizes[7] = {n_q, step ? n_new : 0, step ? n_new : 0, n_c, n_c, n_b, n_b};
  void* dev[7] = {0};
  for (int i = 0; i < 7; ++i) {
    if (!sizes[i]) continue;
    void* host = malloc(sizes[i] * es);
    if (!host || fread(host, es, sizes[i], f) != sizes[i]) { fprintf(stderr, "consumer: short input\n"); return 2; }
    HIP_OK(hipMalloc(&dev[i], sizes[i] * es));
    HIP_OK(hipMemcpy(dev[i], host, sizes[i] * es, hipMemcpyHostToDevice));
    free(host);
  }
  fclose(f);
  float *out = NULL, *lse = NULL;
  void* ws = NULL;
  const size_t ws_bytes = ap_decode_workspace_bytes(B, H, d, T, r, (ap_dtype)dt);
  EXPECT(ws_bytes > 0);
  HIP_OK(hipMalloc((void**)&out, n_q * 4));
  HIP_OK(hipMalloc((void**)&lse, (size_t)B * H * 4));
  HIP_OK(hipMalloc(&ws, ws_bytes));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  const int64_t bstride = shared ? 0 : (int64_t)r * (int64_t)HD;
  ap_status st;
  if (step)
    st = ap_decode_step(dev[0], dev[1], dev[2], dev[3], dev[4], dev[5], dev[6], bstride, NULL, NULL, NULL, NULL, 0,
                        out, lse, NULL, B, H, Hkv, d, T, T_cap, r, sm_scale, (ap_dtype)dt, AP_F32, ws, ws_bytes, stream);
  else
    st = ap_decode_attn(dev[0], dev[3], dev[4], NULL, NULL, dev[5], dev[6], bstride, NULL, NULL, NULL, NULL, 0,
                        out, lse, NULL, B, H, Hkv, d, T, T_cap, r, sm_scale, (ap_dtype)dt, (ap_dtype)dt, AP_F32, ws,
                        ws_bytes, stream);
  if (st != AP_OK) { fprintf(stderr, "consumer: %s: %s\n", ap_status_string(st), ap_last_error()); return 1; }
  HIP_OK(hipStreamSynchronize(stream));
  FILE* g = fopen(out_path, "wb");
  if (!g) { perror(out_path); return 2; }
  float* h_out = (float*)malloc(n_q * 4);
  float* h_lse = (float*)malloc((size_t)B * H * 4);
  HIP_OK(hipMemcpy(h_out, out, n_q * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(h_lse, lse, (size_t)B * H * 4, hipMemcpyDeviceToHost));
  fwrite(h_out, 4, n_q, g);
  fwrite(h_lse, 4, (size_t)B * H, g);
  if (step) {
    char* row = (char*)malloc((size_t)r * es);
    for (int c = 3; c <= 4; ++c)
      for (int b = 0; b < B; ++b) {
        HIP_OK(hipMemcpy(row, (char*)dev[c] + (((size_t)b * T_cap + T - 1) * r) * es, (size_t)r * es,
                         hipMemcpyDeviceToHost));
        fwrite(row, es, r, g);
      }
    free(row);
  }
  fclose(g);
  free(h_out);
  free(h_lse);
  for (int i = 0; i < 7; ++i)
    if (dev[i]) HIP_OK(hipFree(dev[i]));
  HIP_OK(hipFree(out));
  HIP_OK(hipFree(lse));
  HIP_OK(hipFree(ws));
  HIP_OK(hipStreamDestroy(stream));
  printf("consumer: %s done, B=%d H=%d/%d d=%d T=%d r=%d\n", step ? "ap_decode_step" : "ap_decode_attn", B, H, Hkv, d, T, r);
  return 0;
}

int main(int argc, char** argv) {
  if (argc == 2 && strcmp(argv[1], "host") == 0) return host_checks();
  if (argc == 4 && strcmp(argv[1], "run") == 0) return run_case(argv[2], argv[3]);
  fprintf(stderr, "usage: consumer host | consumer run IN.bin OUT.bin\n");
  return 2;
}
