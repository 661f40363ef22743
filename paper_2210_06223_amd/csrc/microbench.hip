// Microbenchmarks that say what this GPU sustains, so that the roofline fractions of the real
// kernels can be read against achievable peaks as well as the data-sheet ones:
//   - bf16 MFMA rate: every SIMD of every CU issues independent v_mfma_f32_16x16x32_bf16 from
//     registers only (no memory traffic), two waves per SIMD;
//   - stream copy: plain out = in over a buffer far larger than the caches, 16 bytes per lane;
//   - weight stream: one 8-wave workgroup per CU, and every one of them reads the same small buffer
//     front to back in 1 KiB wave-wide pieces, as the block kernels read their packed weights: what the
//     L2s deliver when all CUs pull the same lines at once.
// They are launched through the C ABI and timed by the caller with events on its stream.
#include "common.hpp"

namespace lasnet {
namespace {

constexpr int kMfmaPerIter = 16;                 // independent accumulators per wave

__global__ __launch_bounds__(512, 2) void mfma_rate_kernel(int iters, float* __restrict__ sink) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
    b[i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
  }
  floatx4 acc[kMfmaPerIter];
#pragma unroll
  for (int j = 0; j < kMfmaPerIter; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kMfmaPerIter; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kMfmaPerIter; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
  if (s == -1.f) sink[threadIdx.x] = s;          // never true: keeps the loop alive
}

constexpr int kStreamUnroll = 16;                // 16-byte loads a lane keeps in flight

__global__ __launch_bounds__(512, 2) void weight_stream_kernel(const uint4* __restrict__ buf, unsigned pieces,
                                                               int passes, unsigned* __restrict__ sink) {
  // piece = 64 lanes x 16 bytes; wave w of the workgroup takes pieces w, w + 8, ...
  const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned acc = 0;
  for (int p = 0; p < passes; ++p) {
    for (unsigned q0 = wave; q0 < pieces; q0 += 8 * kStreamUnroll) {
      uint4 v[kStreamUnroll];
#pragma unroll
      for (int u = 0; u < kStreamUnroll; ++u) v[u] = buf[(size_t)(q0 + 8 * u) * 64 + lane];   // pieces % 128 == 0
#pragma unroll
      for (int u = 0; u < kStreamUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
  }
  if (acc == 0x9e3779b9u && passes < 0) sink[threadIdx.x] = acc;   // never true: keeps the loads alive
}

}  // namespace
}  // namespace lasnet

using namespace lasnet;

extern "C" {

// Launches the MFMA loop on 2 workgroups of 8 waves per CU; returns the FLOPs the launch performs
// (2 per multiply-add) or 0 on error.  sink: any device buffer of >= 2 KiB (never written).
double lasnet_microbench_mfma(int iters, void* sink, void* hip_stream) {
  if (iters <= 0 || !sink) return 0.0;
  const int grid = device_cu_count() * 2;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(grid), dim3(512), 0, (hipStream_t)hip_stream, iters, (float*)sink);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)grid * 8 /*waves*/ * (double)iters * kMfmaPerIter * (2.0 * 16 * 16 * 32);
}

// One 8-wave workgroup per CU reads buf[0 .. bytes) `passes` times (bytes a multiple of 128 KiB, buf 16-byte
// aligned); returns the bytes the launch reads over all CUs, or 0 on error.
double lasnet_microbench_weight_stream(const void* buf, size_t bytes, int passes, void* sink, void* hip_stream) {
  if (!buf || !sink || passes <= 0 || bytes == 0 || bytes % (128 * 1024) || ((uintptr_t)buf & 15) || bytes > (1u << 30))
    return 0.0;
  const int grid = device_cu_count();
  hipLaunchKernelGGL(weight_stream_kernel, dim3(grid), dim3(512), 0, (hipStream_t)hip_stream, (const uint4*)buf,
                     (unsigned)(bytes / 1024), passes, (unsigned*)sink);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)grid * (double)passes * (double)bytes;
}

// out = in (bytes must be a multiple of 16, pointers 16-byte aligned); returns a lasnet_status.
int lasnet_microbench_copy(const void* in, void* out, size_t bytes, void* hip_stream) {
  if (!in || !out || bytes == 0 || bytes % 16 || (((uintptr_t)in | (uintptr_t)out) & 15)) return LASNET_EINVAL;
  return launch_copy(in, out, bytes, (hipStream_t)hip_stream) == hipSuccess ? LASNET_OK : LASNET_EHIP;
}

}  // extern "C"
