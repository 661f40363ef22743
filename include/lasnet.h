/*
 * liblasnet -- C ABI of the MI355X (gfx950) implementation of the coarse-grained
 * spatially adaptive bottleneck block of "Latency-aware Spatial-wise Dynamic
 * Networks" (LASNet): masker -> active-patch index list -> gather (+1 pixel of
 * neighbours) -> conv1x1 / conv3x3 / conv1x1 -> scatter-add into the residual.
 *
 * Conventions for every entry point
 *   - All pointers are DEVICE pointers unless marked "host".  The caller owns every
 *     buffer; the library allocates nothing that the caller sees and frees nothing (its
 *     one internal buffer is described under "Weight repacking").
 *   - Feature maps are dense NHWC (the channels of one pixel are contiguous).
 *     dtype LASNET_F32: float.  LASNET_BF16: bfloat16 bit patterns (uint16).
 *     Weights have the feature dtype, biases and the masker weights are float.
 *   - BN and the activation are already folded into W*, b* (Sec. 3.4, first paragraph).
 *   - Calls enqueue work on `hip_stream` (a hipStream_t, NULL = default stream) and
 *     return without synchronising.  `count` is read on the device: there is no host
 *     round trip between lasnet_masker and lasnet_sparse_bottleneck.
 *   - Return value: LASNET_OK or a negative lasnet_status.  Arguments are checked, and the
 *     host-side set-up that can fail is done, before the first launch: with any status other than
 *     LASNET_EHIP nothing has been enqueued and no output buffer has been touched.  LASNET_EHIP
 *     reports a failure of the HIP runtime itself (no device, a launch that was refused); the
 *     contents of the output buffers are then unspecified.
 *   - Alignment: none is required.  The matrix-core kernels move 16 bytes per lane, so they
 *     are used only when x, out and the weight buffers are 16-byte aligned (device allocations
 *     are); other pointers are served by the slower shape-generic kernel (lasnet_*_packed, which
 *     has no such fallback, returns LASNET_EUNSUPPORTED).
 *   - A process that has no usable gfx950 device gets LASNET_EHIP from every compute
 *     call; there is no CPU fallback.
 */
#ifndef LASNET_H_
#define LASNET_H_

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define LASNET_API __attribute__((visibility("default")))
#else
#define LASNET_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LASNET_OK = 0,
  LASNET_EINVAL = -1,       /* null pointer, bad dtype, bad S / M                        */
  LASNET_ESHAPE = -2,       /* S does not divide H or W; out shape/dtype differs from x  */
  LASNET_EUNSUPPORTED = -3, /* shape outside what the kernels were built for             */
  LASNET_EALIAS = -4,       /* out aliases x (see lasnet_sparse_bottleneck)              */
  LASNET_EHIP = -5,         /* HIP runtime error (no device, launch failure)             */
  LASNET_ETOOBIG = -6       /* lasnet_sparse_bottleneck_noalloc: the shape's repacked weights
                               exceed LASNET_NOALLOC_MAX_PACKED_BYTES                     */
} lasnet_status;

typedef enum { LASNET_F32 = 0, LASNET_BF16 = 1 } lasnet_dtype;

/* Dense NHWC feature map in device memory: element (n,h,w,c) at ((n*H+h)*W+w)*C+c. */
typedef struct {
  void* data;
  int32_t n, h, w, c;
  int32_t dtype; /* lasnet_dtype */
} lasnet_tensor;

/* Flags for lasnet_sparse_bottleneck_ex / lasnet_dense_bottleneck. */
enum {
  LASNET_POST_RELU = 1,        /* ReLU after the residual add, on active patches only       */
  LASNET_FORCE_GENERIC = 2,    /* use the shape-generic scalar-FMA kernel (fp32 accumulate,
                                  no intermediate rounding) even where an MFMA kernel exists */
  LASNET_SKIP_IDENTITY = 4,    /* caller guarantees out already equals x on inactive patches:
                                  do not copy x to out first                                 */
  LASNET_FORCE_FUSED = 8,      /* run the one-kernel (fused) schedule even where the library would
                                  pick the tiled one (see "Schedules" below); for measurements  */
  LASNET_FORCE_TILED = 16      /* run the three-kernel (tiled) schedule where the shape has one but
                                  the library would pick the fused one; LASNET_EUNSUPPORTED where
                                  it has none, or in lasnet_sparse_bottleneck_noalloc           */
};

LASNET_API int lasnet_version(void);
LASNET_API const char* lasnet_status_string(int status); /* host pointer to a static string */

/*
 * Masker (Sec. 3.2: pooling to the patch grid, then a 1x1 convolution; App. B.1 eq.: one
 * output channel and a strict comparison decide a patch; App. B.1 (2): the masker hands
 * on the list of active patch indices, not a sparse mask).
 *
 *   logit[n,gy,gx] = bm + sum_c Wm[c] * mean_{i,j<S} x[n, gy*S+i, gx*S+j, c]
 *   mask[n,gy,gx]  = logit > thr                  (tie = inactive)
 *   idx            = ascending flat cell ids  n*G*GW + gy*GW + gx  with mask = 1
 *   count[0]       = number of such cells
 *
 * The logit is accumulated in fp64 from the stored x and Wm; the comparison is done in
 * fp64.  x: feature map (f32 or bf16).  Wm: [C] float.  mask: [N*G*GW] bytes (0/1).
 * idx: capacity N*G*GW int32; entries at and beyond count[0] are left untouched.
 * G = H/S, GW = W/S; S must divide H and W (Sec. 3.2 considers divisors only).
 */
LASNET_API int lasnet_masker(const lasnet_tensor* x, const float* Wm, float bm, int S, float thr,
                  uint8_t* mask, int32_t* idx, int32_t* count, void* hip_stream);

/*
 * lasnet_masker with the identity pass-through fused in (Sec. 3.1: positions that are not
 * selected keep the block input; Sec. 3.4 fuses memory-bound operators that share an input --
 * the masker already reads every cell of x).  pass_out: NULL (then exactly lasnet_masker), or
 * a feature map of x's shape and dtype in a different buffer (same buffer: LASNET_EALIAS): every
 * cell whose mask comes out 0 is copied, bit for bit, from x to pass_out; active cells of
 * pass_out are not touched.  Follow with lasnet_sparse_bottleneck_ex / _packed on the same
 * out with LASNET_SKIP_IDENTITY: together they write every element of out exactly once.
 */
LASNET_API int lasnet_masker_ex(const lasnet_tensor* x, const float* Wm, float bm, int S, float thr,
                     uint8_t* mask, int32_t* idx, int32_t* count, lasnet_tensor* pass_out,
                     void* hip_stream);

/* The same fp64 logits as lasnet_masker compares, written out: logits [N*G*GW] double.
 * For calibrating bm/thr on synthetic inputs and for debugging a mask. */
LASNET_API int lasnet_masker_logits(const lasnet_tensor* x, const float* Wm, float bm, int S,
                         double* logits, void* hip_stream);

/*
 * Sparse bottleneck (Sec. 3.1 gather/compute/scatter; Sec. 3.4 and App. B.1 (2),(3):
 * the gather is fused into the dynamic convolution, the scatter into the residual add;
 * Sec. 3.1: positions that are not selected keep the block input).
 *
 * For every cell id in idx[0 .. count[0]) -- cell (n,gy,gx), pixels h in [gy*S, gy*S+S),
 * w in [gx*S, gx*S+S) -- and with y1 taken as 0 outside the image:
 *   y1  = ReLU(b1 + x . W1^T)                          W1 [M][C]
 *   y2  = ReLU(b2 + conv3x3(y1, W2, stride 1, pad 1))  W2 [M][3][3][M] (out,ky,kx,in), cross-correlation
 *   out = x + (b3 + y2 . W3^T)                         W3 [C][M]        no ReLU before the add
 * Every other pixel: out = x, bit for bit.  Neighbour pixels that belong to inactive
 * patches still feed y1 with their true x.  The result does not depend on the order of
 * idx; entries must be unique (not checked).  An entry that is not a cell of this map
 * (negative, or >= N*G*GW) is ignored; a count[0] beyond N*G*GW is read as N*G*GW.
 * idx == NULL means "all cells active" and count is then ignored (may be NULL).
 * The list's STORAGE must have room for N*G*GW entries, as the buffer lasnet_masker fills has: the count is
 * known only on the device, and the kernels may read (never use) entries past count[0] -- they request the
 * list together with the count instead of after it.  A caller that builds its own list pads the buffer.
 *
 * M: bottleneck width.  out: same shape and dtype as x.  Normally a different buffer: in the fused
 * schedule a patch updated in place would corrupt the neighbour read of an adjacent active
 * patch, so out->data == x->data gives LASNET_EALIAS there (and so do buffers that overlap
 * without being the same, on every schedule).  On the tiled schedule (see "Schedules") out may BE x:
 * the block is then updated in place, as App. B.1 (3) stores results into the residual map --
 * inactive patches are simply not touched and no identity copy is made.
 * bf16: products on the matrix cores with fp32 accumulation; y1, y2 are rounded to bf16
 * (nearest even) between the convolutions, out is rounded once after the residual add.
 */
LASNET_API int lasnet_sparse_bottleneck(const lasnet_tensor* x, const int32_t* idx, const int32_t* count,
                             int S, int M,
                             const void* W1, const float* b1,
                             const void* W2, const float* b2,
                             const void* W3, const float* b3,
                             lasnet_tensor* out, void* hip_stream);

/* Same, with LASNET_* flags (see the enum above). */
LASNET_API int lasnet_sparse_bottleneck_ex(const lasnet_tensor* x, const int32_t* idx, const int32_t* count,
                                int S, int M,
                                const void* W1, const float* b1,
                                const void* W2, const float* b2,
                                const void* W3, const float* b3,
                                lasnet_tensor* out, uint32_t flags, void* hip_stream);

/*
 * Schedules.  Two matrix-core schedules exist, and the library picks by shape (Sec. 3.4 discusses
 * this choice of operator fusion against the activation rate; on this GPU the block shape decides):
 *   fused  one kernel: gather + conv1 + conv3x3 + conv3 + scatter-add, y1 and y2 never leave the CU.
 *          Used where a CU can afford to stream all weights per batch of patches (ResNet-101 stages 1-3).
 *   tiled  the paper's own operator split (Sec. 3.4, App. B.1): conv1 over the pixels that some
 *          active patch needs | gather + conv3x3 | conv3 + scatter-add, as three kernels with y1 and
 *          y2 passing through a workspace in device memory.  Built for 1024x256 channels on maps of
 *          up to 196 pixels (14x14) and 2048x512 channels on maps of up to 49 pixels (7x7), any patch
 *          size.  The library's own choice for 2048x512 (measured faster there at every activation
 *          rate); for 1024x256 the fused kernel measured faster or equal at every rate, so the tiled
 *          one runs only with LASNET_FORCE_TILED (a caller that wants the in-place update).
 * Results are the same function of the inputs either way (same roundings: y1, y2 to bf16, out once).
 * The tiled schedule needs lasnet_workspace_bytes() of device memory (that query answers for every
 * shape that has a tiled schedule, chosen by default or not; 0 = none): lasnet_sparse_bottleneck[_ex],
 * lasnet_dense_bottleneck and lasnet_sparse_bottleneck_packed take it from the library's per-stream
 * buffer (see below); lasnet_sparse_bottleneck_planned takes it from the caller;
 * lasnet_sparse_bottleneck_noalloc never uses the tiled schedule.
 */
LASNET_API size_t lasnet_workspace_bytes(int dtype, int N, int H, int W, int C, int M, int S);

/*
 * Weight repacking for the matrix-core kernels.  Those kernels read W1, W2, W3 from ONE
 * buffer in which the weights are laid out fragment by fragment in the order the waves
 * consume them.  lasnet_sparse_bottleneck[_ex] and lasnet_dense_bottleneck take the plain
 * tensors and repack them on every call, on the caller's stream, into device memory the
 * library owns: one buffer per device and stream, allocated with hipMalloc (the only call of
 * these entry points that may block) on first use and again when a shape needs a larger one --
 * the smaller buffer is then kept, not freed, because enqueued work may still read it; at most
 * 8.5 MiB each, all kept until the process ends.  So those entry points cannot be
 * stream-captured before the stream's buffer has its final size.
 * Weights of an inference model do not change, so a caller can instead
 * repack once, like it folded BN once (Sec. 3.4), and pass the result to
 * lasnet_sparse_bottleneck_packed, which allocates nothing:
 *   bytes = lasnet_packed_weights_bytes(dtype, C, M, S)   host query; 0 = this shape has no
 *                                                         matrix-core kernel
 *   lasnet_pack_weights(..., packed, stream)              packed: caller's device buffer
 * The layout depends on (C, M, S); a packed buffer is only valid for the shape it was
 * made for (both schedules read the same layout).  lasnet_sparse_bottleneck_packed is otherwise
 * lasnet_sparse_bottleneck_ex (same semantics, flags LASNET_POST_RELU, LASNET_SKIP_IDENTITY and
 * LASNET_FORCE_FUSED) and returns LASNET_EUNSUPPORTED for shapes or dtypes without a matrix-core
 * kernel.  It allocates nothing on the fused schedule; on the tiled schedule the workspace comes
 * from the library's per-stream buffer (hipMalloc on first use or growth, as above).
 *
 * lasnet_sparse_bottleneck_planned is the fully explicit form, which never allocates: packed
 * weights AND the workspace are the caller's (workspace: 256-byte aligned device memory of at least
 * lasnet_workspace_bytes(); may be NULL when that is 0; LASNET_EINVAL if too small), owned by the
 * call until its work on the stream has finished.  mask: NULL, or the byte mask that lasnet_masker
 * wrote for the same index list (mask[cell] != 0 exactly for the cells in idx[0 .. count[0])); the
 * tiled schedule then reads it instead of scanning the list.
 */
LASNET_API size_t lasnet_packed_weights_bytes(int dtype, int C, int M, int S);
LASNET_API int lasnet_pack_weights(int dtype, int C, int M, int S, const void* W1, const void* W2,
                                   const void* W3, void* packed, void* hip_stream);
LASNET_API int lasnet_sparse_bottleneck_packed(const lasnet_tensor* x, const int32_t* idx,
                                               const int32_t* count, int S, int M,
                                               const void* packed, const float* b1,
                                               const float* b2, const float* b3,
                                               lasnet_tensor* out, uint32_t flags,
                                               void* hip_stream);
LASNET_API int lasnet_sparse_bottleneck_planned(const lasnet_tensor* x, const int32_t* idx,
                                                const int32_t* count, const uint8_t* mask,
                                                int S, int M, const void* packed,
                                                const float* b1, const float* b2, const float* b3,
                                                lasnet_tensor* out, uint32_t flags,
                                                void* workspace, size_t workspace_bytes,
                                                void* hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): lasnet_sparse_bottleneck_ex with the per-call weight
 * repack going to a fixed array in device memory instead of the library's per-stream buffer.
 * This entry point calls no hipMalloc / hipFree and no allocating library routine, on any call.
 *   - The array is LASNET_NOALLOC_MAX_PACKED_BYTES long, exists once per GPU the library runs
 *     on, and is held until the process ends.  Shapes whose repacked weights
 *     (lasnet_packed_weights_bytes) are larger -- the 7x7 stage of ResNet-101, 8.5 MiB -- get
 *     LASNET_ETOOBIG before anything is enqueued; such callers repack once into a buffer of their
 *     own and use lasnet_sparse_bottleneck_packed, which allocates nothing either.
 *   - All calls on one GPU share the array (each call rewrites the part it uses before reading
 *     it, so nothing has to be cleared between calls): calls that overlap on one GPU -- different
 *     streams, or host threads on different streams -- race on it.  Calls on one stream are
 *     ordered and safe.
 *   - Shapes without a matrix-core kernel run the generic kernel, which needs no scratch.
 * Arguments, semantics, flags and results are those of lasnet_sparse_bottleneck_ex, bit for bit.
 */
#define LASNET_NOALLOC_MAX_PACKED_BYTES (4u << 20)
LASNET_API int lasnet_sparse_bottleneck_noalloc(const lasnet_tensor* x, const int32_t* idx,
                                                const int32_t* count, int S, int M,
                                                const void* W1, const float* b1,
                                                const void* W2, const float* b2,
                                                const void* W3, const float* b3,
                                                lasnet_tensor* out, uint32_t flags, void* hip_stream);

/*
 * The static block (activation rate 1, no masker): out = x + F(x) at every pixel -- the
 * l_stat that the paper's latency ratio r_l = l_dyn / l_stat is measured against (Sec. 4.2).
 * Runs the same kernels over tiles that cover the whole map.  flags: LASNET_POST_RELU,
 * LASNET_FORCE_GENERIC, LASNET_FORCE_FUSED, LASNET_FORCE_TILED.
 */
LASNET_API int lasnet_dense_bottleneck(const lasnet_tensor* x, int M,
                            const void* W1, const float* b1,
                            const void* W2, const float* b2,
                            const void* W3, const float* b3,
                            lasnet_tensor* out, uint32_t flags, void* hip_stream);

/* Whether (dtype, C, M, S) has a matrix-core kernel (1) or only the generic one (0);
 * negative status if even the generic kernel cannot take it.  Host-only query. */
LASNET_API int lasnet_has_fast_path(int dtype, int C, int M, int S);

/*
 * Microbenchmarks for the measurement harness (what this GPU sustains, beside the data-sheet peaks the
 * roofline fractions are quoted against).  The caller times them with events on its stream.
 *   lasnet_microbench_mfma   every SIMD issues independent bf16 16x16x32 MFMAs from registers, `iters`
 *                            rounds of 16; returns the FLOPs of the launch (2 per multiply-add), 0 on
 *                            error.  sink: any device buffer of at least 2 KiB (never written).
 *   lasnet_microbench_copy   out = in with the library's copy kernel; bytes a multiple of 16, both
 *                            pointers 16-byte aligned (else LASNET_EINVAL).
 *   lasnet_microbench_weight_stream
 *                            one 8-wave workgroup per CU, each reading buf[0 .. bytes) `passes` times in
 *                            wave-wide 1 KiB pieces, as the block kernels read their packed weights (every CU
 *                            the same lines at the same time); bytes a multiple of 128 KiB, at most 1 GiB, buf
 *                            16-byte aligned; returns the bytes read over all CUs, 0 on error.  sink as above.
 */
LASNET_API double lasnet_microbench_mfma(int iters, void* sink, void* hip_stream);
LASNET_API double lasnet_microbench_weight_stream(const void* buf, size_t bytes, int passes, void* sink,
                                                  void* hip_stream);
LASNET_API int lasnet_microbench_copy(const void* in, void* out, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LASNET_H_ */
