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

// 16-byte streaming store (the destination is not read again by this kernel)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ inline void store_nt16(void* p, const uint4& q) {
  __builtin_nontemporal_store(u32x4{q.x, q.y, q.z, q.w}, reinterpret_cast<u32x4*>(p));
}

// acc += sum over the V elements of one 16-byte piece of x times their masker weights.
__device__ inline void fma_piece(double& acc, const uint4& q, const float4& w0, const float4& w1,
                                 uint16_t /*bf16 tag*/) {
  acc = fma((double)w0.x, (double)bf16_bits_to_float(q.x & 0xffffu), acc);
  acc = fma((double)w0.y, (double)bf16_bits_to_float(q.x >> 16), acc);
  acc = fma((double)w0.z, (double)bf16_bits_to_float(q.y & 0xffffu), acc);
  acc = fma((double)w0.w, (double)bf16_bits_to_float(q.y >> 16), acc);
  acc = fma((double)w1.x, (double)bf16_bits_to_float(q.z & 0xffffu), acc);
  acc = fma((double)w1.y, (double)bf16_bits_to_float(q.z >> 16), acc);
  acc = fma((double)w1.z, (double)bf16_bits_to_float(q.w & 0xffffu), acc);
  acc = fma((double)w1.w, (double)bf16_bits_to_float(q.w >> 16), acc);
}
__device__ inline void fma_piece(double& acc, const uint4& q, const float4& w0, const float4&,
                                 float /*f32 tag*/) {
  acc = fma((double)w0.x, (double)__uint_as_float(q.x), acc);
  acc = fma((double)w0.y, (double)__uint_as_float(q.y), acc);
  acc = fma((double)w0.z, (double)__uint_as_float(q.z), acc);
  acc = fma((double)w0.w, (double)__uint_as_float(q.w), acc);
}

// One wave per cell.  A patch row is one contiguous segment of S*C elements; a wave reads it
// in groups of four 1 KiB pieces (16 bytes per lane each) that are all requested before the
// first one is used, so that enough bytes are in flight to keep HBM busy.
// VEC: 16-byte loads (needs C*sizeof(T) % 16 == 0 and aligned bases).  HOIST: the segment is
// exactly one group (S*C*sizeof(T) == 4 KiB, true for every ResNet stage in bf16), so a lane
// meets the same channels in every row and keeps their masker weights in registers.
template <typename T, bool VEC, bool HOIST>
__global__ __launch_bounds__(kMaskerThreads) void masker_logit_kernel(
    const T* __restrict__ x, const float* __restrict__ Wm, double bm, double thr, int S, int H,
    int W, int C, int G, int GW, int P, uint8_t* __restrict__ mask, double* __restrict__ logits,
    T* __restrict__ pass_out) {
  const int lane = threadIdx.x & 63;
  const int cell = blockIdx.x * kCellsPerBlock + (threadIdx.x >> 6);
  if (cell >= P) return;                      // wave-uniform
  const int n = cell / (G * GW);
  const int rem = cell - n * (G * GW);
  const int gy = rem / GW, gx = rem - gy * GW;
  const int seg = S * C;                      // contiguous elements of one patch row
  const T* cell0 = x + ((size_t)(n * H + gy * S) * W + (size_t)gx * S) * C;
  const size_t pitch = (size_t)W * C;         // elements between patch rows
  double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
  if constexpr (VEC) {
    constexpr int V = 16 / (int)sizeof(T);    // elements per 16-byte piece
    constexpr int GRP = 4 * 64 * V;           // elements per group of four pieces
    if constexpr (HOIST) {
      float4 w[4][2];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = ((lane + 64 * u) * V) % C;
        w[u][0] = *reinterpret_cast<const float4*>(Wm + c);
        w[u][1] = V == 8 ? *reinterpret_cast<const float4*>(Wm + c + 4) : float4{0.f, 0.f, 0.f, 0.f};
      }
      int i = 0;
      for (; i + 2 <= S; i += 2) {            // two rows = eight pieces in flight per lane
        const T* row = cell0 + i * pitch;
        uint4 q[2][4];
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
          for (int u = 0; u < 4; ++u) q[r][u] = *reinterpret_cast<const uint4*>(row + r * pitch + (lane + 64 * u) * V);
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          fma_piece(acc0, q[r][0], w[0][0], w[0][1], T{});
          fma_piece(acc1, q[r][1], w[1][0], w[1][1], T{});
          fma_piece(acc2, q[r][2], w[2][0], w[2][1], T{});
          fma_piece(acc3, q[r][3], w[3][0], w[3][1], T{});
        }
      }
      for (; i < S; ++i) {
        const T* row = cell0 + i * pitch;
        uint4 q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) q[u] = *reinterpret_cast<const uint4*>(row + (lane + 64 * u) * V);
        fma_piece(acc0, q[0], w[0][0], w[0][1], T{});
        fma_piece(acc1, q[1], w[1][0], w[1][1], T{});
        fma_piece(acc2, q[2], w[2][0], w[2][1], T{});
        fma_piece(acc3, q[3], w[3][0], w[3][1], T{});
      }
    } else {
      for (int i = 0; i < S; ++i) {
        const T* row = cell0 + i * pitch;
        int e0 = 0;
        for (; e0 + GRP <= seg; e0 += GRP) {
          uint4 q[4];
          float4 w[4][2];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int e = e0 + (lane + 64 * u) * V, c = e % C;
            q[u] = *reinterpret_cast<const uint4*>(row + e);
            w[u][0] = *reinterpret_cast<const float4*>(Wm + c);
            w[u][1] = V == 8 ? *reinterpret_cast<const float4*>(Wm + c + 4) : float4{0.f, 0.f, 0.f, 0.f};
          }
          fma_piece(acc0, q[0], w[0][0], w[0][1], T{});
          fma_piece(acc1, q[1], w[1][0], w[1][1], T{});
          fma_piece(acc2, q[2], w[2][0], w[2][1], T{});
          fma_piece(acc3, q[3], w[3][0], w[3][1], T{});
        }
        for (int e = e0 + lane * V; e < seg; e += 64 * V) {      // pieces left over
          const int c = e % C;
          const uint4 q = *reinterpret_cast<const uint4*>(row + e);
          const float4 w0 = *reinterpret_cast<const float4*>(Wm + c);
          const float4 w1 = V == 8 ? *reinterpret_cast<const float4*>(Wm + c + 4) : float4{0.f, 0.f, 0.f, 0.f};
          fma_piece(acc0, q, w0, w1, T{});
        }
      }
    }
  } else {
    for (int i = 0; i < S; ++i) {
      const T* row = cell0 + i * pitch;
      for (int e = lane; e < seg; e += 64) {
        const int c = e % C;
        if constexpr (sizeof(T) == 2) acc0 = fma((double)Wm[c], (double)bf16_bits_to_float(row[e]), acc0);
        else acc0 = fma((double)Wm[c], (double)row[e], acc0);
      }
    }
  }
  // the butterfly leaves the same bits in every lane (a + b == b + a), so the decision is wave-uniform
  const double acc = wave_sum((acc0 + acc1) + (acc2 + acc3));
  const double logit = bm + acc / (double)(S * S);
  const bool on = logit > thr;
  if (lane == 0) {
    if (logits) logits[cell] = logit;
    if (mask) mask[cell] = on ? 1 : 0;
  }
  // Identity pass-through fused into the masker (Sec. 3.1: positions that are not selected keep
  // the input): a cell that stays inactive is copied now, while its rows are still in cache.
  if (pass_out != nullptr && !on) {
    T* out0 = pass_out + (cell0 - x);
    if constexpr (VEC) {
      constexpr int V = 16 / (int)sizeof(T);
      constexpr int GRP = 4 * 64 * V;
      for (int i = 0; i < S; ++i) {
        const T* row = cell0 + i * pitch;
        T* orow = out0 + i * pitch;
        int e = lane * V;
        if (HOIST && i + 2 <= S) {            // two whole rows = eight pieces in flight per lane
          uint4 q[2][4];
#pragma unroll
          for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int u = 0; u < 4; ++u) q[r][u] = *reinterpret_cast<const uint4*>(row + r * pitch + e + u * 64 * V);
#pragma unroll
          for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int u = 0; u < 4; ++u)
              store_nt16(orow + r * pitch + e + u * 64 * V, q[r][u]);
          ++i;
          continue;
        }
        for (; e + GRP - 64 * V < seg; e += GRP) {
          uint4 q[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) q[u] = *reinterpret_cast<const uint4*>(row + e + u * 64 * V);
#pragma unroll
          for (int u = 0; u < 4; ++u) store_nt16(orow + e + u * 64 * V, q[u]);
        }
        for (; e < seg; e += 64 * V) *reinterpret_cast<uint4*>(orow + e) = *reinterpret_cast<const uint4*>(row + e);
      }
    } else {
      for (int i = 0; i < S; ++i) {
        const T* row = cell0 + i * pitch;
        T* orow = out0 + i * pitch;
        for (int e = lane; e < seg; e += 64) orow[e] = row[e];
      }
    }
  }
}

// The common case (a patch row is exactly 4 KiB, S in {1, 2, 4, 8}: every ResNet stage in bf16) with the
// cell split by rows over WPC waves of the workgroup: a wave takes two rows (8 KiB, eight 16-byte
// pieces per lane), keeps them in registers, and the waves of a cell add their partial sums in a
// fixed order through LDS.  An inactive cell is then written to pass_out from those registers: x is
// read once, and because a wave's share is small and there are WPC times more waves, the reading of
// some cells overlaps the writing of others (with a whole 32 KiB cell per wave, all waves first
// read, then all wrote: the two halves of the traffic did not overlap).
template <typename T, int WPC, int RPW = 2>
__global__ __launch_bounds__(kMaskerThreads) void masker_rows_kernel(
    const T* __restrict__ x, const float* __restrict__ Wm, double bm, double thr, int H, int W,
    int C, int G, int GW, int P, uint8_t* __restrict__ mask, double* __restrict__ logits,
    T* __restrict__ pass_out) {
  constexpr int S = RPW * WPC;              // RPW rows per wave
  constexpr int V = 16 / (int)sizeof(T);
  constexpr int CPB = kCellsPerBlock / WPC;   // cells per workgroup
  __shared__ double part[kCellsPerBlock];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cell = blockIdx.x * CPB + wave / WPC, sub = wave % WPC;
  const bool valid = cell < P;                // wave-uniform; every wave reaches the barrier
  const int cc = valid ? cell : 0;
  const int n = cc / (G * GW);
  const int rem = cc - n * (G * GW);
  const int gy = rem / GW, gx = rem - gy * GW;
  const size_t pitch = (size_t)W * C;
  const size_t off = ((size_t)(n * H + gy * S + RPW * sub) * W + (size_t)gx * S) * C + (size_t)lane * V;
  uint4 q[RPW][4];
#pragma unroll
  for (int r = 0; r < RPW; ++r)
#pragma unroll
    for (int u = 0; u < 4; ++u) q[r][u] = *reinterpret_cast<const uint4*>(x + off + r * pitch + u * 64 * V);
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int c = ((lane + 64 * u) * V) % C;
    const float4 w0 = *reinterpret_cast<const float4*>(Wm + c);
    const float4 w1 = V == 8 ? *reinterpret_cast<const float4*>(Wm + c + 4) : float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < RPW; ++r) fma_piece(acc[u], q[r][u], w0, w1, T{});
  }
  double tot = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
  if constexpr (WPC > 1) {
    if (lane == 0) part[wave] = tot;
    __syncthreads();
    tot = 0.0;
#pragma unroll
    for (int k = 0; k < WPC; ++k) tot += part[wave / WPC * WPC + k];   // the same order in every wave of the cell
  }
  const double logit = bm + tot / (double)(S * S);
  const bool on = logit > thr;
  if (!valid) return;
  if (lane == 0 && sub == 0) {
    if (logits) logits[cell] = logit;
    if (mask) mask[cell] = on ? 1 : 0;
  }
  if (pass_out != nullptr && !on) {
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
      for (int u = 0; u < 4; ++u) store_nt16(pass_out + off + r * pitch + u * 64 * V, q[r][u]);
  }
}

// Ordered stream compaction by one workgroup.  A thread takes V consecutive cells (one 8-byte
// load when V = 8), a shuffle scan over the per-thread counts gives each thread its rank
// inside its wave, a scan over the 16 wave totals its rank inside the 1024*V-cell round, and
// a running base its rank overall.  Integer work only: the list is the ascending sequence
// of active cell ids whatever the timing.
constexpr int kCompactThreads = 1024;

template <int V>
__global__ __launch_bounds__(kCompactThreads) void compact_kernel(
    const uint8_t* __restrict__ mask, int P, int32_t* __restrict__ idx,
    int32_t* __restrict__ count) {
  __shared__ int wave_tot[kCompactThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int base = 0;                                // identical in every thread
  for (int start = 0; start < P; start += kCompactThreads * V) {
    const int i0 = start + tid * V;
    unsigned on = 0;                           // bit b: cell i0 + b is active
    if constexpr (V == 8) {
      if (i0 + 8 <= P) {
        const unsigned long long q = *reinterpret_cast<const unsigned long long*>(mask + i0);
#pragma unroll
        for (int b = 0; b < 8; ++b) on |= ((q >> (8 * b)) & 0xffull) != 0 ? (1u << b) : 0u;
      } else {
        for (int b = 0; b < 8; ++b)
          if (i0 + b < P && mask[i0 + b] != 0) on |= 1u << b;
      }
    } else {
      on = (i0 < P && mask[i0] != 0) ? 1u : 0u;
    }
    const int c = __popc(on);
    int incl = c;                              // inclusive scan over the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(incl, o, 64);
      if (lane >= o) incl += t;
    }
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int k = 0; k < kCompactThreads / 64; ++k) {
      const int t = wave_tot[k];
      before += (k < wv) ? t : 0;
      total += t;
    }
    int pos = base + before + incl - c;
    while (on) {
      const int b = __ffs(on) - 1;
      idx[pos++] = i0 + b;
      on &= on - 1;
    }
    base += total;
    __syncthreads();                           // wave_tot is rewritten next round
  }
  if (tid == 0) *count = base;
}

}  // namespace

hipError_t launch_masker(const lasnet_tensor& x, const float* Wm, float bm, int S, float thr,
                         uint8_t* mask, int32_t* idx, int32_t* count, double* logits,
                         void* pass_out, hipStream_t st) {
  const int G = x.h / S, GW = x.w / S, P = x.n * G * GW;
  const dim3 grid(P > 0 ? (P + kCellsPerBlock - 1) / kCellsPerBlock : 1), block(kMaskerThreads);
  const size_t esz = x.dtype == LASNET_BF16 ? 2 : 4;
  const bool vec = ((size_t)x.c * esz) % 16 == 0 && ((uintptr_t)x.data % 16) == 0 &&
                   ((uintptr_t)Wm % 16) == 0 && (x.c % 8 == 0) && ((uintptr_t)pass_out % 16) == 0;
  const bool hoist = vec && (size_t)S * x.c * esz == 4096;   // one group of four pieces per patch row
#define LASNET_MASKER_LAUNCH(T, VEC, HOIST)                                                   \
  hipLaunchKernelGGL((masker_logit_kernel<T, VEC, HOIST>), grid, block, 0, st, (const T*)x.data, \
                     Wm, (double)bm, (double)thr, S, x.h, x.w, x.c, G, GW, P, mask, logits,      \
                     (T*)pass_out)
#define LASNET_MASKER_ROWS(T, WPC, ...)                                                          \
  hipLaunchKernelGGL((masker_rows_kernel<T, WPC, ##__VA_ARGS__>), dim3((P + kCellsPerBlock / WPC - 1) / (kCellsPerBlock / WPC)), \
                     block, 0, st, (const T*)x.data, Wm, (double)bm, (double)thr, x.h, x.w, x.c, G, GW, P,     \
                     mask, logits, (T*)pass_out)
  if (P == 0) {
    // empty batch: nothing to pool; the compaction below still writes count = 0
  } else if (hoist && (S == 1 || S == 2 || S == 4 || S == 8)) {
    if (x.dtype == LASNET_BF16) {
      if (S == 1) LASNET_MASKER_ROWS(uint16_t, 1, 1);      // pixel-level cells (7x7x2048): a cell is one row
      else if (S == 2) LASNET_MASKER_ROWS(uint16_t, 2, 1); // one row per wave: 0.9 us faster than two at stage 3
      else if (S == 4 && pass_out) LASNET_MASKER_ROWS(uint16_t, 4, 1);   // with the pass-through: 1.3 us faster
      else if (S == 4) LASNET_MASKER_ROWS(uint16_t, 2);                  // without: 0.7 us faster
      else LASNET_MASKER_ROWS(uint16_t, 4);
    } else {
      if (S == 1) LASNET_MASKER_ROWS(float, 1, 1);
      else if (S == 2) LASNET_MASKER_ROWS(float, 2, 1);
      else if (S == 4) LASNET_MASKER_ROWS(float, 2);
      else LASNET_MASKER_ROWS(float, 4);
    }
  } else if (x.dtype == LASNET_BF16) {
    if (hoist) LASNET_MASKER_LAUNCH(uint16_t, true, true);
    else if (vec) LASNET_MASKER_LAUNCH(uint16_t, true, false);
    else LASNET_MASKER_LAUNCH(uint16_t, false, false);
  } else {
    if (hoist) LASNET_MASKER_LAUNCH(float, true, true);
    else if (vec) LASNET_MASKER_LAUNCH(float, true, false);
    else LASNET_MASKER_LAUNCH(float, false, false);
  }
#undef LASNET_MASKER_LAUNCH
#undef LASNET_MASKER_ROWS
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (count) {
    if (((uintptr_t)mask % 8) == 0)
      hipLaunchKernelGGL(compact_kernel<8>, dim3(1), dim3(kCompactThreads), 0, st, mask, P, idx, count);
    else
      hipLaunchKernelGGL(compact_kernel<1>, dim3(1), dim3(kCompactThreads), 0, st, mask, P, idx, count);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace lasnet
