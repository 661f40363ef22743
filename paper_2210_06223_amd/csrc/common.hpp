// Shared declarations of liblasnet's translation units (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "lasnet.h"

namespace lasnet {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Geometry of one call, by value into every kernel.
struct Geom {
  int N, H, W, C, M, S;
  int G, GW;       // patch grid: G = H/S rows, GW = W/S columns
  int P;           // N*G*GW cells
};

struct BlockWeights {
  const void* W1; const float* b1;
  const void* W2; const float* b2;
  const void* W3; const float* b3;
};

// ---- launchers (each returns a hipError_t from the launch, never synchronises) ----
hipError_t launch_masker(const lasnet_tensor& x, const float* Wm, float bm, int S, float thr,
                         uint8_t* mask, int32_t* idx, int32_t* count, double* logits,
                         void* pass_out, hipStream_t st);

hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st);

// Generic scalar-FMA kernel: any C, M; S limited by LDS. Returns hipErrorInvalidValue if
// the tile does not fit in LDS.
bool generic_fits(int M, int S);
hipError_t launch_generic(int dtype, const Geom& g, const void* x, const int32_t* idx,
                          const int32_t* count, const BlockWeights& w, void* out, bool post_relu,
                          hipStream_t st);

// One matrix-core instantiation: its shape and its two launchers.
struct MfmaVariant {
  int C, M, S;
  size_t packed_bytes;
  size_t max_map_bytes;      // largest feature map the kernel addresses (0 = no limit of its own)
  hipError_t (*prepare)();   // host-side set-up that can fail (per-device kernel attributes); enqueues nothing
  hipError_t (*pack)(const void* W1, const void* W2, const void* W3, void* packed, hipStream_t st);
  hipError_t (*launch)(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                       const void* packed, const float* b1, const float* b2, const float* b3,
                       void* out, bool post_relu, hipStream_t st);
};
int device_cu_count();

// The tiled schedule (three kernels, y1 and y2 through a workspace) of one (C, M); any patch size.
// It reads the same packed weight buffer as the fused kernels of that (C, M).
struct TiledVariant {
  int C, M;
  bool preferred;                               // the library's own choice for this shape (else only on request)
  bool (*takes)(const Geom& g);                 // does the map fit its image groups?
  size_t (*workspace_bytes)(const Geom& g);
  hipError_t (*prepare)();
  hipError_t (*launch)(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                       const uint8_t* cellmask, const void* packed, const float* b1, const float* b2,
                       const float* b3, void* out, bool post_relu, void* workspace, hipStream_t st);
};
// The tiled variant that takes this call, or nullptr (then the fused kernel runs).
const TiledVariant* find_tiled(const Geom& g);

// Matrix-core kernel: only for the (C, M, S) it was instantiated for.  It reads the three
// weight tensors from one buffer of mfma_packed_bytes() that launch_pack() fills.
bool mfma_supported(int C, int M, int S);
size_t mfma_max_map_bytes(int C, int M, int S);
hipError_t prepare_mfma(int C, int M, int S);
hipError_t prepare_generic(int dtype);
size_t mfma_packed_bytes(int C, int M, int S);
hipError_t launch_pack(int C, int M, int S, const void* W1, const void* W2, const void* W3,
                       void* packed, hipStream_t st);
hipError_t launch_mfma(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                       const void* packed, const float* b1, const float* b2, const float* b3,
                       void* out, bool post_relu, hipStream_t st);

}  // namespace lasnet
