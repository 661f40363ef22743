// Shape-generic sparse bottleneck (any C and M, fp32 or bf16 storage) on the vector ALUs,
// and the identity copy for inactive patches.  One workgroup per active patch: gather the
// (S+2)x(S+2) window straight from NHWC global memory while computing conv1 (Sec. 3.4,
// gather fused into the dynamic convolution), keep y1 and y2 in LDS as fp32, add the
// residual and write the S x S result in place of the patch (scatter fused with the add).
// This is the correctness path for shapes without a matrix-core kernel (and all of fp32):
// fp32 accumulation, no intermediate rounding.
#include "common.hpp"

namespace lasnet {
namespace {

constexpr int kGenThreads = 256;
constexpr size_t kLdsLimit = 160 * 1024 - 1024;

template <typename T> __device__ inline float ld(const T* p);
template <> __device__ inline float ld<float>(const float* p) { return *p; }
template <> __device__ inline float ld<uint16_t>(const uint16_t* p) {
  return __uint_as_float(((uint32_t)*p) << 16);
}
template <typename T> __device__ inline void st(T* p, float v);
template <> __device__ inline void st<float>(float* p, float v) { *p = v; }
template <> __device__ inline void st<uint16_t>(uint16_t* p, float v) {
  const __bf16 b = (__bf16)v;                 // round to nearest even
  *p = __builtin_bit_cast(uint16_t, b);
}

template <typename T>
__global__ __launch_bounds__(kGenThreads) void bneck_generic_kernel(
    Geom g, const T* __restrict__ x, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ count, const T* __restrict__ W1, const float* __restrict__ b1,
    const T* __restrict__ W2, const float* __restrict__ b2, const T* __restrict__ W3,
    const float* __restrict__ b3, T* __restrict__ out, int post_relu) {
  extern __shared__ float lds[];
  const int S = g.S, Tw = S + 2, WW = Tw * Tw, M = g.M, C = g.C;
  float* y1 = lds;                 // [WW][M]
  float* y2 = lds + (size_t)WW * M;  // [S*S][M]
  const int nact = idx ? min(*count, g.P) : g.P;
  for (int e = blockIdx.x; e < nact; e += gridDim.x) {
    const int cell = idx ? idx[e] : e;
    if ((unsigned)cell >= (unsigned)g.P) continue;           // not a cell of this map (uniform over the workgroup)
    const int n = cell / (g.G * g.GW);
    const int rem = cell - n * (g.G * g.GW);
    const int gy = rem / g.GW, gx = rem - gy * g.GW;
    // conv1 + ReLU on the window; 0 outside the image (zero padding of conv1's output)
    for (int t = threadIdx.x; t < WW * M; t += kGenThreads) {
      const int r = t / M, m = t - r * M;
      const int h = gy * S + r / Tw - 1, w = gx * S + r % Tw - 1;
      float v = 0.f;
      if (h >= 0 && h < g.H && w >= 0 && w < g.W) {
        const T* xp = x + ((size_t)(n * g.H + h) * g.W + w) * C;
        const T* wp = W1 + (size_t)m * C;
        float a = b1[m];
        for (int c = 0; c < C; ++c) a = fmaf(ld(xp + c), ld(wp + c), a);
        v = fmaxf(a, 0.f);
      }
      y1[t] = v;
    }
    __syncthreads();
    // conv2 3x3 + ReLU on the S x S interior
    for (int t = threadIdx.x; t < S * S * M; t += kGenThreads) {
      const int q = t / M, o = t - q * M;
      const int i = q / S, j = q - i * S;
      float a = b2[o];
      for (int ky = 0; ky < 3; ++ky)
        for (int kx = 0; kx < 3; ++kx) {
          const float* src = y1 + (size_t)((i + ky) * Tw + (j + kx)) * M;
          const T* wp = W2 + ((size_t)(o * 3 + ky) * 3 + kx) * M;
          for (int m = 0; m < M; ++m) a = fmaf(src[m], ld(wp + m), a);
        }
      y2[t] = fmaxf(a, 0.f);
    }
    __syncthreads();
    // conv3 + residual add, stored at the patch's own position
    for (int t = threadIdx.x; t < S * S * C; t += kGenThreads) {
      const int q = t / C, c = t - q * C;
      const int i = q / S, j = q - i * S;
      const float* src = y2 + (size_t)q * M;
      const T* wp = W3 + (size_t)c * M;
      float a = b3[c];
      for (int o = 0; o < M; ++o) a = fmaf(src[o], ld(wp + o), a);
      const size_t off = ((size_t)(n * g.H + gy * S + i) * g.W + (gx * S + j)) * C + c;
      float r = ld(x + off) + a;
      if (post_relu) r = fmaxf(r, 0.f);
      st(out + off, r);
    }
    __syncthreads();   // y1/y2 are reused by the next patch of this workgroup
  }
}

// out = x, 16 bytes per lane, grid-stride; the byte tail (if any) by the first lanes.
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src,
                                                   uint4* __restrict__ dst, size_t n16,
                                                   const uint8_t* __restrict__ tsrc,
                                                   uint8_t* __restrict__ tdst, int tail) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
    dst[i] = src[i];
  if (blockIdx.x == 0 && (int)threadIdx.x < tail) tdst[threadIdx.x] = tsrc[threadIdx.x];
}

size_t generic_lds_bytes(int M, int S) {
  return ((size_t)(S + 2) * (S + 2) + (size_t)S * S) * M * sizeof(float);
}

}  // namespace

bool generic_fits(int M, int S) { return generic_lds_bytes(M, S) <= kLdsLimit; }

hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st_) {
  if (bytes == 0) return hipSuccess;
  if (((uintptr_t)src | (uintptr_t)dst) % 16 != 0)
    return hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st_);
  const size_t n16 = bytes / 16;
  const int tail = (int)(bytes - n16 * 16);
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st_, (const uint4*)src,
                     (uint4*)dst, n16, (const uint8_t*)src + n16 * 16, (uint8_t*)dst + n16 * 16,
                     tail);
  return hipGetLastError();
}

// The kernels take up to kLdsLimit bytes of dynamic LDS: said once per device and kernel.
hipError_t prepare_generic(int dtype) {
  static std::atomic<unsigned long long> done[2];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const int which = dtype == LASNET_BF16 ? 1 : 0;
  const unsigned long long bit = dev < 64 ? 1ull << dev : 0ull;
  if (done[which].load(std::memory_order_acquire) & bit) return hipSuccess;
  const void* k = which ? (const void*)bneck_generic_kernel<uint16_t> : (const void*)bneck_generic_kernel<float>;
  e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) done[which].fetch_or(bit, std::memory_order_release);
  return e;
}

hipError_t launch_generic(int dtype, const Geom& g, const void* x, const int32_t* idx,
                          const int32_t* count, const BlockWeights& w, void* out, bool post_relu,
                          hipStream_t st_) {
  if (g.P == 0) return hipSuccess;
  const size_t lds = generic_lds_bytes(g.M, g.S);
  if (lds > kLdsLimit) return hipErrorInvalidValue;
  if (hipError_t e = prepare_generic(dtype); e != hipSuccess) return e;
  const int grid = g.P < 256 * 16 ? g.P : 256 * 16;
  if (dtype == LASNET_BF16) {
    hipLaunchKernelGGL(bneck_generic_kernel<uint16_t>, dim3(grid), dim3(kGenThreads), lds, st_, g,
                       (const uint16_t*)x, idx, count, (const uint16_t*)w.W1, w.b1, (const uint16_t*)w.W2,
                       w.b2, (const uint16_t*)w.W3, w.b3, (uint16_t*)out, (int)post_relu);
  } else {
    hipLaunchKernelGGL(bneck_generic_kernel<float>, dim3(grid), dim3(kGenThreads), lds, st_, g,
                       (const float*)x, idx, count, (const float*)w.W1, w.b1, (const float*)w.W2, w.b2,
                       (const float*)w.W3, w.b3, (float*)out, (int)post_relu);
  }
  return hipGetLastError();
}

}  // namespace lasnet
