// extern "C" boundary of liblasnet: argument validation and kernel dispatch only.
#include "common.hpp"

#include <map>
#include <mutex>
#include <utility>

using namespace lasnet;

namespace {

// Device memory the library owns: one buffer per (device, stream) for the repacked weights
// of calls that pass raw W1/W2/W3.  Work on one stream is ordered, so calls on the same stream
// may share it; calls on different streams get different buffers.  A buffer that turns out too
// small is not freed (work already enqueued may still read it): a larger one is allocated beside
// it and the old one is kept until the process ends.  Shapes with a matrix-core kernel need at
// most 8.5 MiB, so what accumulates is bounded by a few buffers of that size per stream.
struct Workspace { void* ptr = nullptr; size_t cap = 0; };
std::mutex g_ws_mu;
std::map<std::pair<int, hipStream_t>, Workspace> g_ws;

void* get_workspace(hipStream_t st, size_t bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return nullptr;
  std::lock_guard<std::mutex> lock(g_ws_mu);
  Workspace& w = g_ws[std::make_pair(dev, st)];
  if (w.cap < bytes) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    w.ptr = p;                                   // the previous buffer, if any, stays allocated
    w.cap = bytes;
  }
  return w.ptr;
}

// Repacked weights for callers that cannot allocate (lasnet_sparse_bottleneck_noalloc): a fixed
// array in device memory, one copy per GPU the library runs on, held until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: the address that
// kernels and copies take is the one that call returns, looked up once per device.
static __device__ __align__(256) unsigned char scratch[LASNET_NOALLOC_MAX_PACKED_BYTES];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];                // per device; nullptr = not looked up yet
std::mutex g_scratch_mu;

void* scratch_for_current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

bool device_ok() {
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || n <= 0) {
    (void)hipGetLastError();
    return false;
  }
  return true;
}

int check_tensor(const lasnet_tensor* t) {
  if (!t) return LASNET_EINVAL;
  if (t->dtype != LASNET_F32 && t->dtype != LASNET_BF16) return LASNET_EINVAL;
  if (t->n < 0 || t->h <= 0 || t->w <= 0 || t->c <= 0) return LASNET_ESHAPE;
  if (t->n > 0 && !t->data) return LASNET_EINVAL;
  // pixel indices are 32-bit inside the kernels
  if ((long long)t->n * t->h * t->w >= (1ll << 31)) return LASNET_EUNSUPPORTED;
  return LASNET_OK;
}

// Tile side for the static block: the largest of the built S that divides H and W for
// this (C, M); otherwise the largest divisor the generic kernel can hold in LDS.
int dense_tile(int dtype, int H, int W, int C, int M, bool force_generic) {
  if (dtype == LASNET_BF16 && !force_generic)
    for (int s = 16; s >= 1; --s)
      if (H % s == 0 && W % s == 0 && mfma_supported(C, M, s)) return s;
  for (int s = 16; s >= 1; --s)
    if (H % s == 0 && W % s == 0 && generic_fits(M, s)) return s;
  return 0;
}

// How a block call gets the device memory it needs beyond its arguments.
struct Scratchpad {
  bool fixed_array = false;        // raw weights are repacked into this device's `scratch` array (no allocation)
  bool from_caller = false;        // `workspace` / `workspace_bytes` are the caller's
  void* workspace = nullptr;
  size_t workspace_bytes = 0;
  const uint8_t* cellmask = nullptr;   // the masker's byte mask of the same list, if the caller passes it
};

Geom make_geom(const lasnet_tensor* x, int M, int S) {
  Geom g;
  g.N = x->n; g.H = x->h; g.W = x->w; g.C = x->c; g.M = M; g.S = S;
  g.G = x->h / S; g.GW = x->w / S; g.P = x->n * g.G * g.GW;
  return g;
}

size_t round256(size_t v) { return (v + 255) / 256 * 256; }

// packed != nullptr: the caller passes repacked weights (W1..W3 unused).
int run_block(const lasnet_tensor* x, const int32_t* idx, const int32_t* count, int S, int M,
              const void* W1, const float* b1, const void* W2, const float* b2, const void* W3,
              const float* b3, const void* packed, lasnet_tensor* out, uint32_t flags, bool dense,
              void* stream, const Scratchpad& pad = Scratchpad()) {
  int s = check_tensor(x);
  if (s != LASNET_OK) return s;
  if (!out) return LASNET_EINVAL;
  s = check_tensor(out);
  if (s != LASNET_OK) return s;
  if (!b1 || !b2 || !b3) return LASNET_EINVAL;
  if (!packed && (!W1 || !W2 || !W3)) return LASNET_EINVAL;
  if (M <= 0) return LASNET_EINVAL;
  if (!dense && idx && !count) return LASNET_EINVAL;
  if (out->n != x->n || out->h != x->h || out->w != x->w || out->c != x->c ||
      out->dtype != x->dtype)
    return LASNET_ESHAPE;
  const bool force_generic = (flags & LASNET_FORCE_GENERIC) != 0;
  if (dense) {
    S = dense_tile(x->dtype, x->h, x->w, x->c, M, force_generic);
    if (S == 0) return LASNET_EUNSUPPORTED;
  }
  if (S <= 0) return LASNET_EINVAL;
  if (x->h % S != 0 || x->w % S != 0) return LASNET_ESHAPE;
  const size_t map_bytes = (size_t)x->n * x->h * x->w * x->c * (x->dtype == LASNET_BF16 ? 2 : 4);
  // The matrix-core kernels move 16 bytes per lane: x, out and the packed weights must be 16-byte
  // aligned for them (C is a multiple of 64 there, so every pixel then is).  Anything else, and maps
  // beyond a kernel's own addressing limit, go to the generic kernel.
  bool fast = x->dtype == LASNET_BF16 && !force_generic && mfma_supported(x->c, M, S);
  if (fast) {
    const size_t lim = mfma_max_map_bytes(x->c, M, S);
    uintptr_t low = (uintptr_t)x->data | (uintptr_t)out->data | (uintptr_t)packed;
    if (!packed) low |= (uintptr_t)W1 | (uintptr_t)W2 | (uintptr_t)W3;     // the repack reads 16-byte pieces
    if ((low & 15) != 0 || (lim != 0 && map_bytes > lim)) fast = false;
  }
  if (packed && !fast) return LASNET_EUNSUPPORTED;
  if (!fast && !generic_fits(M, S)) return LASNET_EUNSUPPORTED;
  if (fast && !packed && pad.fixed_array && mfma_packed_bytes(x->c, M, S) > sizeof(scratch))
    return LASNET_ETOOBIG;
  const Geom g = make_geom(x, M, S);
  // Deep stages run the tiled schedule (three kernels, y1 and y2 through a workspace) unless the
  // caller asks for the fused kernel or cannot give or allow a workspace.
  const TiledVariant* tiled = nullptr;
  if (fast && !(flags & LASNET_FORCE_FUSED) && !pad.fixed_array) {
    tiled = find_tiled(g);
    if (tiled && !tiled->preferred && !(flags & LASNET_FORCE_TILED)) tiled = nullptr;
  }
  if ((flags & LASNET_FORCE_TILED) && !tiled) return LASNET_EUNSUPPORTED;
  // out == x (update in place, as App. B.1 (3) stores into the residual map) is safe only on the tiled
  // schedule: its last kernel reads and writes nothing but the active pixels' own elements, after the
  // kernel that reads neighbours has finished.  In one kernel a patch updated in place would corrupt a
  // neighbouring patch's window.  Buffers that overlap without being the same are never accepted.
  const bool in_place = x->n > 0 && out->data == x->data;
  if (x->n > 0 && !in_place) {
    const uintptr_t a = (uintptr_t)x->data, b = (uintptr_t)out->data;
    if (a < b + map_bytes && b < a + map_bytes) return LASNET_EALIAS;
  }
  if (in_place && !tiled) return LASNET_EALIAS;
  const size_t packed_need = (fast && !packed) ? round256(mfma_packed_bytes(x->c, M, S)) : 0;
  const size_t tiled_need = tiled ? tiled->workspace_bytes(g) : 0;
  if (pad.from_caller && tiled && (!pad.workspace || pad.workspace_bytes < tiled_need || ((uintptr_t)pad.workspace & 255)))
    return LASNET_EINVAL;
  if (!device_ok()) return LASNET_EHIP;
  if (x->n == 0) return LASNET_OK;

  const BlockWeights w{W1, b1, W2, b2, W3, b3};
  hipStream_t st = (hipStream_t)stream;
  // Everything that can fail on the host comes before the first launch: kernel attributes, then the
  // memory for the repacked weights and the tiled schedule's intermediates (the caller's, the
  // library's per stream, or `scratch`).
  hipError_t e = !fast ? prepare_generic(x->dtype) : tiled ? tiled->prepare() : prepare_mfma(x->c, M, S);
  if (e != hipSuccess) return LASNET_EHIP;
  unsigned char* tiled_ws = nullptr;
  if (pad.from_caller) {
    tiled_ws = (unsigned char*)pad.workspace;              // (this entry takes packed weights: packed_need is 0)
  } else if (pad.fixed_array) {
    if (packed_need) {
      void* p = scratch_for_current_device();
      if (!p) return LASNET_EHIP;
      e = launch_pack(x->c, M, S, W1, W2, W3, p, st);
      if (e != hipSuccess) return LASNET_EHIP;
      packed = p;
    }
  } else if (packed_need + tiled_need) {
    unsigned char* ws = (unsigned char*)get_workspace(st, packed_need + tiled_need);
    if (!ws) return LASNET_EHIP;
    if (packed_need) {
      e = launch_pack(x->c, M, S, W1, W2, W3, ws, st);
      if (e != hipSuccess) return LASNET_EHIP;
      packed = ws;
    }
    tiled_ws = ws + packed_need;
  }
  if (!dense && idx && !in_place && !(flags & LASNET_SKIP_IDENTITY)) {
    e = launch_copy(x->data, out->data, map_bytes, st);
    if (e != hipSuccess) return LASNET_EHIP;
  }
  const bool relu = (flags & LASNET_POST_RELU) != 0;
  if (tiled)
    e = tiled->launch(g, x->data, idx, count, idx ? pad.cellmask : nullptr, packed, b1, b2, b3, out->data, relu,
                      tiled_ws, st);
  else if (fast)
    e = launch_mfma(g, x->data, idx, count, packed, b1, b2, b3, out->data, relu, st);
  else
    e = launch_generic(x->dtype, g, x->data, idx, count, w, out->data, relu, st);
  return e == hipSuccess ? LASNET_OK : LASNET_EHIP;
}

int masker_common(const lasnet_tensor* x, const float* Wm, float bm, int S, float thr,
                  uint8_t* mask, int32_t* idx, int32_t* count, double* logits,
                  const lasnet_tensor* pass_out, void* stream) {
  int s = check_tensor(x);
  if (s != LASNET_OK) return s;
  if (!Wm) return LASNET_EINVAL;
  if (S <= 0) return LASNET_EINVAL;
  if (x->h % S != 0 || x->w % S != 0) return LASNET_ESHAPE;
  if (pass_out) {
    s = check_tensor(pass_out);
    if (s != LASNET_OK) return s;
    if (pass_out->n != x->n || pass_out->h != x->h || pass_out->w != x->w || pass_out->c != x->c ||
        pass_out->dtype != x->dtype)
      return LASNET_ESHAPE;
    if (x->n > 0 && pass_out->data == x->data) return LASNET_EALIAS;
  }
  if (!device_ok()) return LASNET_EHIP;
  const hipError_t e = launch_masker(*x, Wm, bm, S, thr, mask, idx, count, logits,
                                     pass_out ? pass_out->data : nullptr, (hipStream_t)stream);
  return e == hipSuccess ? LASNET_OK : LASNET_EHIP;
}

}  // namespace

extern "C" {

int lasnet_version(void) { return 100; }

const char* lasnet_status_string(int status) {
  switch (status) {
    case LASNET_OK: return "ok";
    case LASNET_EINVAL: return "invalid argument (null pointer, bad dtype, S or M)";
    case LASNET_ESHAPE: return "shape mismatch (S must divide H and W; out must match x)";
    case LASNET_EUNSUPPORTED: return "shape not supported by the built kernels";
    case LASNET_EALIAS: return "out must not alias x (only the tiled schedule can update x in place)";
    case LASNET_EHIP: return "HIP runtime error or no gfx950 device";
    case LASNET_ETOOBIG: return "repacked weights exceed the fixed scratch array of lasnet_sparse_bottleneck_noalloc";
    default: return "unknown status";
  }
}

int lasnet_masker(const lasnet_tensor* x, const float* Wm, float bm, int S, float thr,
                  uint8_t* mask, int32_t* idx, int32_t* count, void* hip_stream) {
  if (!count) return LASNET_EINVAL;
  const bool empty = x && x->n == 0;            // an empty batch has no mask or idx storage
  if (!empty && (!mask || !idx)) return LASNET_EINVAL;
  return masker_common(x, Wm, bm, S, thr, mask, idx, count, nullptr, nullptr, hip_stream);
}

int lasnet_masker_ex(const lasnet_tensor* x, const float* Wm, float bm, int S, float thr,
                     uint8_t* mask, int32_t* idx, int32_t* count, lasnet_tensor* pass_out,
                     void* hip_stream) {
  if (!count) return LASNET_EINVAL;
  const bool empty = x && x->n == 0;
  if (!empty && (!mask || !idx)) return LASNET_EINVAL;
  return masker_common(x, Wm, bm, S, thr, mask, idx, count, nullptr, pass_out, hip_stream);
}

int lasnet_masker_logits(const lasnet_tensor* x, const float* Wm, float bm, int S, double* logits,
                         void* hip_stream) {
  if (!logits) return LASNET_EINVAL;
  return masker_common(x, Wm, bm, S, 0.f, nullptr, nullptr, nullptr, logits, nullptr, hip_stream);
}

int lasnet_sparse_bottleneck_ex(const lasnet_tensor* x, const int32_t* idx, const int32_t* count,
                                int S, int M, const void* W1, const float* b1, const void* W2,
                                const float* b2, const void* W3, const float* b3,
                                lasnet_tensor* out, uint32_t flags, void* hip_stream) {
  return run_block(x, idx, count, S, M, W1, b1, W2, b2, W3, b3, nullptr, out, flags, false,
                   hip_stream);
}

size_t lasnet_packed_weights_bytes(int dtype, int C, int M, int S) {
  if (dtype != LASNET_BF16 || C <= 0 || M <= 0 || S <= 0) return 0;
  return mfma_packed_bytes(C, M, S);
}

int lasnet_pack_weights(int dtype, int C, int M, int S, const void* W1, const void* W2,
                        const void* W3, void* packed, void* hip_stream) {
  if (!W1 || !W2 || !W3 || !packed) return LASNET_EINVAL;
  if (lasnet_packed_weights_bytes(dtype, C, M, S) == 0) return LASNET_EUNSUPPORTED;
  if (!device_ok()) return LASNET_EHIP;
  return launch_pack(C, M, S, W1, W2, W3, packed, (hipStream_t)hip_stream) == hipSuccess ? LASNET_OK
                                                                                         : LASNET_EHIP;
}

int lasnet_sparse_bottleneck_packed(const lasnet_tensor* x, const int32_t* idx, const int32_t* count,
                                    int S, int M, const void* packed, const float* b1,
                                    const float* b2, const float* b3, lasnet_tensor* out,
                                    uint32_t flags, void* hip_stream) {
  if (!packed) return LASNET_EINVAL;
  return run_block(x, idx, count, S, M, nullptr, b1, nullptr, b2, nullptr, b3, packed, out,
                   flags & ~(uint32_t)LASNET_FORCE_GENERIC, false, hip_stream);
}

size_t lasnet_workspace_bytes(int dtype, int N, int H, int W, int C, int M, int S) {
  if (dtype != LASNET_BF16 || N <= 0 || H <= 0 || W <= 0 || C <= 0 || M <= 0 || S <= 0 || H % S || W % S) return 0;
  if (!mfma_supported(C, M, S)) return 0;
  lasnet_tensor t{nullptr, N, H, W, C, dtype};
  const Geom g = make_geom(&t, M, S);
  const TiledVariant* tv = find_tiled(g);
  return tv ? tv->workspace_bytes(g) : 0;
}

int lasnet_sparse_bottleneck_planned(const lasnet_tensor* x, const int32_t* idx, const int32_t* count,
                                     const uint8_t* mask, int S, int M, const void* packed,
                                     const float* b1, const float* b2, const float* b3,
                                     lasnet_tensor* out, uint32_t flags, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
  if (!packed) return LASNET_EINVAL;
  Scratchpad pad;
  pad.from_caller = true;
  pad.workspace = workspace;
  pad.workspace_bytes = workspace_bytes;
  pad.cellmask = mask;
  return run_block(x, idx, count, S, M, nullptr, b1, nullptr, b2, nullptr, b3, packed, out,
                   flags & ~(uint32_t)LASNET_FORCE_GENERIC, false, hip_stream, pad);
}

int lasnet_sparse_bottleneck(const lasnet_tensor* x, const int32_t* idx, const int32_t* count, int S,
                             int M, const void* W1, const float* b1, const void* W2,
                             const float* b2, const void* W3, const float* b3, lasnet_tensor* out,
                             void* hip_stream) {
  return run_block(x, idx, count, S, M, W1, b1, W2, b2, W3, b3, nullptr, out, 0u, false, hip_stream);
}

int lasnet_sparse_bottleneck_noalloc(const lasnet_tensor* x, const int32_t* idx, const int32_t* count,
                                     int S, int M, const void* W1, const float* b1, const void* W2,
                                     const float* b2, const void* W3, const float* b3,
                                     lasnet_tensor* out, uint32_t flags, void* hip_stream) {
  Scratchpad fixed;
  fixed.fixed_array = true;
  return run_block(x, idx, count, S, M, W1, b1, W2, b2, W3, b3, nullptr, out, flags, false,
                   hip_stream, fixed);
}

int lasnet_dense_bottleneck(const lasnet_tensor* x, int M, const void* W1, const float* b1,
                            const void* W2, const float* b2, const void* W3, const float* b3,
                            lasnet_tensor* out, uint32_t flags, void* hip_stream) {
  return run_block(x, nullptr, nullptr, 0, M, W1, b1, W2, b2, W3, b3, nullptr, out,
                   flags & (LASNET_POST_RELU | LASNET_FORCE_GENERIC | LASNET_FORCE_FUSED | LASNET_FORCE_TILED), true,
                   hip_stream);
}

int lasnet_has_fast_path(int dtype, int C, int M, int S) {
  if (dtype != LASNET_F32 && dtype != LASNET_BF16) return LASNET_EINVAL;
  if (C <= 0 || M <= 0 || S <= 0) return LASNET_EINVAL;
  if (dtype == LASNET_BF16 && mfma_supported(C, M, S)) return 1;
  return generic_fits(M, S) ? 0 : LASNET_EUNSUPPORTED;
}

}  // extern "C"
