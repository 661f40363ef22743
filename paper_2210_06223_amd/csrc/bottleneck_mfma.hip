// Dispatch over the matrix-core instantiations (one table per mfma_stage*.hip).
#include "common.hpp"

namespace lasnet {

const MfmaVariant* mfma_variants_stage1(int* n);
const MfmaVariant* mfma_variants_stage2(int* n);
const MfmaVariant* mfma_variants_stage3(int* n);
const MfmaVariant* mfma_variants_stage4(int* n);

namespace {
const MfmaVariant* find_variant(int C, int M, int S) {
  const MfmaVariant* (*tables[])(int*) = {mfma_variants_stage1, mfma_variants_stage2, mfma_variants_stage3,
                                          mfma_variants_stage4};
  for (auto get : tables) {
    int n = 0;
    const MfmaVariant* t = get(&n);
    for (int i = 0; i < n; ++i)
      if (t[i].C == C && t[i].M == M && t[i].S == S) return &t[i];
  }
  return nullptr;
}
}  // namespace

const TiledVariant* tiled_variants(int* n);

const TiledVariant* find_tiled(const Geom& g) {
  int n = 0;
  const TiledVariant* t = tiled_variants(&n);
  for (int i = 0; i < n; ++i)
    if (t[i].C == g.C && t[i].M == g.M && t[i].takes(g)) return &t[i];
  return nullptr;
}

int device_cu_count() {
  static std::atomic<int> cached[64];         // per device; 0 = not asked yet
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (dev >= 0 && dev < 64 && (n = cached[dev].load(std::memory_order_relaxed)) > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
  if (dev >= 0 && dev < 64) cached[dev].store(n, std::memory_order_relaxed);
  return n;
}

bool mfma_supported(int C, int M, int S) { return find_variant(C, M, S) != nullptr; }

size_t mfma_max_map_bytes(int C, int M, int S) {
  const MfmaVariant* v = find_variant(C, M, S);
  return v ? v->max_map_bytes : 0;
}

hipError_t prepare_mfma(int C, int M, int S) {
  const MfmaVariant* v = find_variant(C, M, S);
  return v ? v->prepare() : hipErrorInvalidValue;
}

size_t mfma_packed_bytes(int C, int M, int S) {
  const MfmaVariant* v = find_variant(C, M, S);
  return v ? v->packed_bytes : 0;
}

hipError_t launch_pack(int C, int M, int S, const void* W1, const void* W2, const void* W3,
                       void* packed, hipStream_t st) {
  const MfmaVariant* v = find_variant(C, M, S);
  return v ? v->pack(W1, W2, W3, packed, st) : hipErrorInvalidValue;
}

hipError_t launch_mfma(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                       const void* packed, const float* b1, const float* b2, const float* b3,
                       void* out, bool post_relu, hipStream_t st) {
  if (g.P == 0) return hipSuccess;
  const MfmaVariant* v = find_variant(g.C, g.M, g.S);
  return v ? v->launch(g, x, idx, count, packed, b1, b2, b3, out, post_relu, st) : hipErrorInvalidValue;
}

}  // namespace lasnet
