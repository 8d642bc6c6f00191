// Measurement aid, not part of the method: a plain streaming read of a device buffer, the
// yardstick the bandwidth-bound kernels of this library are held against on the machine they
// run on (the nominal HBM peak is not reachable by any kernel; this one shows what is).
#include "ap_common.hpp"

namespace ap {
namespace {

constexpr int kProbeWgs = 2048;         // eight workgroups per CU
constexpr int kProbeUnroll = 8;         // 16-byte loads in flight per thread

// grid kProbeWgs, 256 threads: workgroup w reads chunks [w * per, (w + 1) * per) of 16 bytes,
// `per` a multiple of 256 * kProbeUnroll.  The XOR of everything a wave read goes to
// sink[4 w + wave], so the loads cannot be dropped.
// NT: the loads carry the non-temporal hint (a stream that is read once).
template <bool NT>
__global__ void __launch_bounds__(256)
stream_read(const u32x4_t* __restrict__ src, uint32_t* __restrict__ sink, size_t per) {
  const u32x4_t* p = src + (size_t)blockIdx.x * per;
  u32x4_t acc = {0, 0, 0, 0};
  for (size_t i = threadIdx.x; i < per; i += 256 * kProbeUnroll) {
    u32x4_t v[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) v[u] = NT ? __builtin_nontemporal_load(p + i + u * 256) : p[i + u * 256];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u];
  }
  uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
  if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = x;
}

}  // namespace

size_t probe_read_granule() { return (size_t)kProbeWgs * 256 * kProbeUnroll * 16; }

ap_status launch_probe_read(const void* src, size_t bytes, uint32_t* sink, bool non_temporal, hipStream_t stream) {
  const size_t per = bytes / 16 / kProbeWgs;
  if (non_temporal)
    hipLaunchKernelGGL(stream_read<true>, dim3(kProbeWgs), dim3(256), 0, stream, (const u32x4_t*)src, sink, per);
  else
    hipLaunchKernelGGL(stream_read<false>, dim3(kProbeWgs), dim3(256), 0, stream, (const u32x4_t*)src, sink, per);
  return check_launch("ap_probe_read");
}

}  // namespace ap
