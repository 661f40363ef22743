// Masker: per-patch average pool -> 1x1 conv to one logit -> strict threshold (Sec. 3.2,
// App. B.1 equation), then an ordered compaction of the mask into the active-patch index
// list (App. B.1 (2)).  HBM-bound: reads x once, 16 bytes per lane per load.
#include "common.hpp"

namespace lasnet {
namespace {

constexpr int kMaskerThreads = 256;          // 4 waves, one patch cell per wave
constexpr int kCellsPerBlock = kMaskerThreads / 64;

__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ inline float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// One wave per cell.  VEC = true: 16-byte loads (needs C*sizeof(T) % 16 == 0, aligned base).
template <typename T, bool VEC>
__global__ __launch_bounds__(kMaskerThreads) void masker_logit_kernel(
    const T* __restrict__ x, const float* __restrict__ Wm, double bm, double thr, int S, int H,
    int W, int C, int G, int GW, int P, uint8_t* __restrict__ mask, double* __restrict__ logits) {
  const int lane = threadIdx.x & 63;
  const int cell = blockIdx.x * kCellsPerBlock + (threadIdx.x >> 6);
  if (cell >= P) return;                      // wave-uniform
  const int n = cell / (G * GW);
  const int rem = cell - n * (G * GW);
  const int gy = rem / GW, gx = rem - gy * GW;
  constexpr int V = VEC ? (16 / (int)sizeof(T)) : 1;
  const int seg = S * C;                      // contiguous elements of one patch row
  double acc = 0.0;
  for (int i = 0; i < S; ++i) {
    const T* row = x + ((size_t)(n * H + gy * S + i) * W + (size_t)gx * S) * C;
    for (int e = lane * V; e < seg; e += 64 * V) {
      const int c = e % C;
      if constexpr (VEC && sizeof(T) == 2) {
        const uint4 q = *reinterpret_cast<const uint4*>(row + e);
        const float4 w0 = *reinterpret_cast<const float4*>(Wm + c);
        const float4 w1 = *reinterpret_cast<const float4*>(Wm + c + 4);
        acc = fma((double)w0.x, (double)bf16_bits_to_float(q.x & 0xffffu), acc);
        acc = fma((double)w0.y, (double)bf16_bits_to_float(q.x >> 16), acc);
        acc = fma((double)w0.z, (double)bf16_bits_to_float(q.y & 0xffffu), acc);
        acc = fma((double)w0.w, (double)bf16_bits_to_float(q.y >> 16), acc);
        acc = fma((double)w1.x, (double)bf16_bits_to_float(q.z & 0xffffu), acc);
        acc = fma((double)w1.y, (double)bf16_bits_to_float(q.z >> 16), acc);
        acc = fma((double)w1.z, (double)bf16_bits_to_float(q.w & 0xffffu), acc);
        acc = fma((double)w1.w, (double)bf16_bits_to_float(q.w >> 16), acc);
      } else if constexpr (VEC && sizeof(T) == 4) {
        const float4 q = *reinterpret_cast<const float4*>(row + e);
        const float4 w0 = *reinterpret_cast<const float4*>(Wm + c);
        acc = fma((double)w0.x, (double)q.x, acc);
        acc = fma((double)w0.y, (double)q.y, acc);
        acc = fma((double)w0.z, (double)q.z, acc);
        acc = fma((double)w0.w, (double)q.w, acc);
      } else if constexpr (sizeof(T) == 2) {
        acc = fma((double)Wm[c], (double)bf16_bits_to_float(row[e]), acc);
      } else {
        acc = fma((double)Wm[c], (double)row[e], acc);
      }
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) {
    const double logit = bm + acc / (double)(S * S);
    if (logits) logits[cell] = logit;
    if (mask) mask[cell] = logit > thr ? 1 : 0;
  }
}

// Ordered stream compaction by one workgroup: wave ballot + popcount gives each active
// cell its rank inside its wave, a scan over the 16 wave totals its rank inside the
// 1024-cell chunk, and a running base its rank overall.  Integer work only: the list is
// the ascending sequence of active cell ids whatever the timing.
constexpr int kCompactThreads = 1024;

__global__ __launch_bounds__(kCompactThreads) void compact_kernel(
    const uint8_t* __restrict__ mask, int P, int32_t* __restrict__ idx,
    int32_t* __restrict__ count) {
  __shared__ int wave_tot[kCompactThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int base = 0;                                // identical in every thread
  for (int start = 0; start < P; start += kCompactThreads) {
    const int i = start + tid;
    const bool on = (i < P) && (mask[i] != 0);
    const unsigned long long b = __ballot(on);
    const int rank = __popcll(b & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wv] = __popcll(b);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int k = 0; k < kCompactThreads / 64; ++k) {
      const int t = wave_tot[k];
      before += (k < wv) ? t : 0;
      total += t;
    }
    if (on) idx[base + before + rank] = i;
    base += total;
    __syncthreads();                           // wave_tot is rewritten next round
  }
  if (tid == 0) *count = base;
}

}  // namespace

hipError_t launch_masker(const lasnet_tensor& x, const float* Wm, float bm, int S, float thr,
                         uint8_t* mask, int32_t* idx, int32_t* count, double* logits,
                         hipStream_t st) {
  const int G = x.h / S, GW = x.w / S, P = x.n * G * GW;
  const dim3 grid(P > 0 ? (P + kCellsPerBlock - 1) / kCellsPerBlock : 1), block(kMaskerThreads);
  const size_t esz = x.dtype == LASNET_BF16 ? 2 : 4;
  const bool vec = ((size_t)x.c * esz) % 16 == 0 && ((uintptr_t)x.data % 16) == 0 &&
                   ((uintptr_t)Wm % 16) == 0 && (x.c % 8 == 0);
#define LASNET_MASKER_LAUNCH(T, VEC)                                                          \
  hipLaunchKernelGGL((masker_logit_kernel<T, VEC>), grid, block, 0, st, (const T*)x.data, Wm, \
                     (double)bm, (double)thr, S, x.h, x.w, x.c, G, GW, P, mask, logits)
  if (P == 0) {
    // empty batch: nothing to pool; the compaction below still writes count = 0
  } else if (x.dtype == LASNET_BF16) {
    if (vec) LASNET_MASKER_LAUNCH(uint16_t, true); else LASNET_MASKER_LAUNCH(uint16_t, false);
  } else {
    if (vec) LASNET_MASKER_LAUNCH(float, true); else LASNET_MASKER_LAUNCH(float, false);
  }
#undef LASNET_MASKER_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (count) {
    hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(kCompactThreads), 0, st, mask, P, idx, count);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace lasnet
