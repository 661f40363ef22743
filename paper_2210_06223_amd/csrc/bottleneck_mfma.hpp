// Fused sparse bottleneck on the gfx950 matrix cores (bf16 in, fp32 accumulate): the kernel
// templates.  Each mfma_stage*.hip instantiates them for the shapes of one ResNet stage.
//
// One workgroup owns a run of consecutive entries of the active-patch index list (at most
// PPW patches at a time) and runs the whole block for them without leaving the CU (Sec. 3.4
// / App. B.1: gather fused into the dynamic convolution, scatter fused into the residual
// add; here the three convolutions are fused as well, so packed patches never go back to
// memory):
//
//   phase 0  decode the cell ids; collect the pixels of all (S+2)x(S+2) windows into a set
//            (LDS hash table): a pixel shared by the windows of neighbouring patches gets
//            ONE row, pixels outside the image get none -- the overlapping neighbour area
//            of Sec. 3.4 is loaded and convolved once per workgroup, not once per patch
//   phase 1  conv1 over the U unique rows: x rows stream through LDS in KC-channel chunks
//            (2-4 chunks requested ahead), y1 = ReLU(W1 x + b1) -> LDS
//   phase 2  conv2: implicit GEMM over the 9 taps, y1 rows looked up per window position
//            (an all-zero row stands for "outside the image") -> y2 in LDS
//   phase 3  conv3 + b3 + residual x, rounded once, stored at the patch's own pixels
//
// Every GEMM is computed transposed, D[channel][pixel] = W[channel][k] * act[pixel][k], with
// v_mfma_f32_16x16x32_bf16.  The weight fragment (A operand) is read straight from global
// memory / L2, from a buffer that pack_weights_kernel has laid out fragment by fragment in
// the order the waves consume them; the activation fragment (B operand) comes from LDS.
// In the result a lane holds 4 consecutive rows = channels; which channel sits in which row
// of which tile is chosen (lane_channel) so that a lane's results are runs of 8 consecutive
// channels and four lanes cover 64 contiguous bytes of a pixel.
// Waves are arranged WR x WC (pixel-blocks x channel-blocks) per phase.
#pragma once
#include "common.hpp"

#include <type_traits>

namespace lasnet {
namespace {

__device__ inline floatx4 mfma16(bf16x8 a, bf16x8 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

constexpr int cdiv(int a, int b) { return (a + b - 1) / b; }
constexpr int cmax(int a, int b) { return a > b ? a : b; }
constexpr int roundup(int a, int b) { return cdiv(a, b) * b; }
constexpr int pow2_at_least(int v) { int p = 1; while (p < v) p *= 2; return p; }

// C, M, S: block shape.  PPW: patches per batch (max).  R1MAX: rows of y1 kept in LDS (unique
// window pixels of a batch; a batch is cut short if it would need more).  NSTG: LDS stages of
// the x stream (KC channels each; x chunks are in flight NSTG-1 chunks ahead).  WRi x WCi:
// wave grid of conv i.  RD2/RD3: k-steps of weights a wave keeps in flight in conv2/conv3.
// NB3: channel tiles per conv3 pass.
template <int C_, int M_, int S_, int PPW_, int R1MAX_, int NW_, int KC_, int NSTG_, int WR1_,
          int WC1_, int WR2_, int WC2_, int RD2_, int WR3_, int WC3_, int NB3_, int RD3_>
struct Cfg {
  static constexpr int C = C_, M = M_, S = S_, PPW = PPW_, NW = NW_, KC = KC_, NSTG = NSTG_;
  static constexpr int NT = NW * 64;
  static constexpr int T = S + 2, WW = T * T;
  static constexpr int R1MAX = R1MAX_, R1B = R1MAX / 16;
  static constexpr int ZROW = R1MAX;                   // index of the all-zero y1 row
  static constexpr int WR1 = WR1_, WC1 = WC1_, NBW1 = M / 16 / WC1;
  static constexpr int WR2 = WR2_, WC2 = WC2_, NBW2 = M / 16 / WC2, RD2 = RD2_;
  static constexpr int WR3 = WR3_, WC3 = WC3_, NBT3 = C / 16 / WC3, NB3 = NB3_, RD3 = RD3_;
  static constexpr int R2 = PPW * S * S;
  static constexpr int R2B = roundup(cdiv(R2, 16), cmax(WR2, WR3)), R2P = R2B * 16;
  static constexpr int NB3ROWS = 4 * WR3;              // row blocks conv3 takes at a time
  // LDS rows have power-of-two pitch and their 16-byte chunks are XOR-swizzled (see swz()):
  // measured on gfx950, ds_read_b128 then runs at ~6 clk per wave against ~9 with a padded pitch.
  static constexpr int LDX = KC, LDY = M;
  static constexpr int XMASK = KC / 8 - 1;
  static constexpr int YMASK = LDY / 8 - 1 < 15 ? LDY / 8 - 1 : 15;   // swizzle key bits of a y1/y2 row
  static constexpr int MS = M / 32;                    // k-steps over the mid channels
  static constexpr int LDY2 = LDY, YMASK2 = YMASK;     // pitch / key bits of the y2 rows conv2 writes
  // the packed weight buffers: bytes from one k-step's fragments to the next, and sizes
  static constexpr int WD = 2;                         // conv1's weight ring, in chunks
  static constexpr bool Y1_IN_XS = false;              // y1s is a region of its own
  static constexpr bool ACTS_BARRIER = false;          // conv2 / conv3 find their LDS inputs complete on entry
  static constexpr bool Y1_TO_GLOBAL = false, Y2_TO_GLOBAL = false;   // conv1 / conv2 results stay in LDS
  static constexpr int W_KSTEP_BYTES = M * 64;
  static constexpr unsigned W1_BYTES = M * C * 2, W2_BYTES = 9 * M * M * 2, W3_BYTES = C * M * 2;
  static constexpr int HT = pow2_at_least(cmax(2 * R1MAX, PPW * (S + 2) * (S + 2) + 1));  // hash table slots
  // LDS map (bytes)
  static constexpr int OFF_HKEY = 0;                            // int  [HT]     pixel+1 or 0
  static constexpr int OFF_HVAL = OFF_HKEY + HT * 4;            // short[HT]     row of that pixel
  static constexpr int OFF_WINROW = OFF_HVAL + HT * 2;          // short[PPW*WW] row of each window position
  static constexpr int OFF_ROWPIX = (OFF_WINROW + PPW * WW * 2 + 15) / 16 * 16;  // int[R1MAX]
  static constexpr int OFF_PIXQ = OFF_ROWPIX + R1MAX * 4;       // int  [R2P]
  static constexpr int OFF_MISC = OFF_PIXQ + R2P * 4;           // int  [4]
  static constexpr int OFF_CELL = OFF_MISC + 16;                // int  [PPW]    cell ids of the batch
  static constexpr int OFF_BIAS = (OFF_CELL + PPW * 4 + 15) / 16 * 16;   // float[M | M | C]: b1, b2, b3
  static constexpr int OFF_Y1 = OFF_BIAS + (2 * M + C) * 4;
  static constexpr int Y1_BYTES = (R1MAX + 1) * LDY * 2;
  static constexpr int OFF_XS = OFF_Y1 + Y1_BYTES;
  static constexpr int STAGE_ELEMS = R1MAX * LDX;
  static constexpr int XS_BYTES = NSTG * STAGE_ELEMS * 2 + 1024;  // + 1 KiB that padding loads land in
  static constexpr int Y2_BYTES = R2P * LDY * 2;
  static constexpr int LDS_BYTES = OFF_XS + cmax(XS_BYTES, Y2_BYTES);
  static constexpr size_t PACKED_ELEMS = (size_t)M * C * 2 + 9 * (size_t)M * M;
  static_assert(R1MAX % 16 == 0 && R1MAX >= WW && R1MAX < 32767, "y1 rows");
  static_assert(R1B % WR1 == 0, "conv1 row blocks split evenly over the wave rows");
  static_assert(HT > PPW * WW, "the hash table always keeps an empty slot, so probing ends");
  static_assert(WR1 * WC1 == NW && WR2 * WC2 == NW && WR3 * WC3 == NW, "wave grid");
  static_assert(M % (16 * WC1) == 0 && M % (16 * WC2) == 0 && C % (16 * WC3) == 0, "channel split");
  static_assert(NBT3 % NB3 == 0 && NB3 % 2 == 0, "conv3 passes; 16-byte epilogue pieces");
  static_assert(C % (2 * KC) == 0 && KC == 64 && M % 32 == 0, "k steps");
  // x stream: chunk c lives in stage c % NSTG.  XD chunks are requested ahead of the one being
  // consumed: all of them when they all fit, else one less than there are stages (a stage is
  // refilled right after the barrier that follows its last read).
  static constexpr int NCH = C / KC;
  static constexpr int XD = NCH <= NSTG ? NCH : NSTG - 1;
  static_assert(NSTG >= 3 && XD >= 2, "x stream depth");
  static_assert(LDY % 64 == 0 && (LDY & (LDY - 1)) == 0, "y rows: power-of-two pitch, whole swizzle groups");
  static_assert((9 * MS) % RD2 == 0 && MS % RD3 == 0, "weight rings");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  // Waves a SIMD holds when the CU is full of these workgroups: the register budget per wave
  // is 512 / that (a 4-wave workgroup alone on its CU may use the accumulation registers too).
  static constexpr int WAVES_PER_SIMD = cmax(1, ((160 * 1024) / LDS_BYTES) * NW / 4);
  static_assert(NW * 2048 <= R1MAX * LDY * 2, "conv3's per-wave transpose areas sit in the y1 rows below the zero row");
};

// Pointers into global memory and LDS carry explicit address spaces: through generic pointers
// every LDS access would need a conversion and every weight load would be a FLAT load, which
// also counts on lgkmcnt and so would be waited for with each LDS read.  The phase functions
// are inlined into the kernel by default (a real call saves and restores half of the vector
// registers through scratch memory on every call).
#ifndef LASNET_PHASE_INLINE
#define LASNET_PHASE_INLINE __attribute__((always_inline))
#endif
#define AS_GLOBAL __attribute__((address_space(1)))
#define AS_LDS __attribute__((address_space(3)))
typedef const AS_GLOBAL void* gptr_t;
typedef AS_LDS void* lptr_t;
typedef const AS_GLOBAL __bf16* g_bf16_p;      // read-only global bf16
typedef const AS_GLOBAL float* g_f32_p;
typedef AS_LDS __bf16* l_bf16_p;
typedef const AS_LDS __bf16* l_bf16_cp;
typedef const AS_LDS int* l_i32_cp;
typedef const AS_LDS short* l_i16_cp;
typedef const AS_LDS float* l_f32_cp;

// Element offset of 16-byte chunk `chunk` in an LDS row of pitch `ld` elements whose chunks
// are XOR-swizzled with `key` (low 4 bits of the chunk index at most).
__device__ inline int swz(int row, int ld, int chunk, int key, int mask = 15) {
  return row * ld + ((chunk ^ (key & mask)) << 3);
}

// The same address for the B-fragment reads of the k-loops, split so that the part that changes
// with the k-step is a compile-time constant: chunk = 4*s + lg never carries, so
// (4*s + lg) ^ key = (4*s) ^ (lg ^ key), and in bytes the fragment of k-step s sits at
//   row_bytes + ((64*s) ^ key_bytes),   key_bytes = (lg ^ (key & mask)) << 4.
// One xor-add per read and two registers per row, instead of one register per (row, k-step).
struct FragRow { int row_bytes, key_bytes; };
__device__ __forceinline__ FragRow frag_row(int row, int ld, int lg, int key, int mask = 15) {
  return FragRow{row * ld * 2, (lg ^ (key & mask)) << 4};
}
__device__ __forceinline__ bf16x8 frag_read(const AS_LDS __bf16* base, FragRow r, int s) {
  int key = r.key_bytes;
  // opaque to the optimiser: otherwise (64*s) ^ key is computed for every s ahead of the loop,
  // kept in registers across the whole phase, and some of them end up spilled
  asm volatile("" : "+v"(key));
  return *reinterpret_cast<const AS_LDS bf16x8*>(reinterpret_cast<const AS_LDS char*>(base) + r.row_bytes +
                                                 ((64 * s) ^ key));
}

// Which output channel a lane holds.  In the 16x16 result of an MFMA, lane group lg (= lane / 16)
// holds rows 4*lg .. 4*lg+3 in its 4 accumulator elements v.  A pass computes nb tiles (j) of
// 16 channels each; which channel is row i of tile j is free (the weights are repacked to
// match), and it is chosen so that what a lane holds of tiles 2t and 2t+1 are 8 consecutive
// channels, and the four lane groups together 32 consecutive ones:
//   channel = base + 32*(j/2) + 8*lg + 4*(j%2) + v            (nb even)
// One 16-byte store per lane then writes 64 contiguous bytes per pixel (whole HBM bursts),
// and the same 16 bytes are one swizzle chunk of an LDS row.  nb odd: base + 4*nb*lg + 4*j + v.
__host__ __device__ inline int lane_channel(int base, int nb, int j, int lg, int v) {
  return (nb & 1) ? base + lg * (4 * nb) + j * 4 + v
                  : base + (j >> 1) * 32 + lg * 8 + (j & 1) * 4 + v;
}
// Channel whose weights sit in A-operand row i (0..15) of tile j.
__host__ __device__ inline int arow_channel(int base, int nb, int j, int i) {
  return lane_channel(base, nb, j, i >> 2, i & 3);
}

__device__ inline unsigned hash_pix(int pix) { return ((unsigned)pix * 2654435761u) >> 12; }

// Wave-uniform value -> scalar register, so that the compiler branches on it with scalar
// branches instead of exec masks.
__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
// The value, behind a barrier the optimiser cannot look through.  Each phase derives its lane
// addresses from a fresh copy of the thread id: derived from the kernel's one copy they are all
// hoisted to the kernel's top, where some forty of them stay live across every phase and push the
// k-loops' weight rings into scratch memory (a reload from there in the middle of a k-loop also
// waits for every weight load requested before it).
__device__ __forceinline__ int opaque(int v) {
  asm volatile("" : "+v"(v));
  return v;
}

// Calls f(integral_constant<n>) for the run-time n in [LO, HI]: the row-block count of a
// phase becomes a compile-time constant, so each phase's inner loop is straight-line code.
template <int LO, int HI, class F>
__device__ __forceinline__ void dispatch_count(int n, F&& f) {
  if constexpr (LO >= HI) {
    f(std::integral_constant<int, HI>{});
  } else {
    if (n <= LO) f(std::integral_constant<int, LO>{});
    else dispatch_count<LO + 1, HI>(n, static_cast<F&&>(f));
  }
}

// Workgroup barrier that waits for this wave's LDS traffic and for all but the youngest VM
// of its global-memory operations -- NOT for all of them, as __syncthreads() would: the
// x chunks and weights already requested for later steps stay in flight across it.
// Built with LASNET_DRAIN_AT_BARRIERS (the check build of the library) every such barrier waits for
// ALL of the wave's global-memory operations instead: slower, and independent of the hand-made
// count.  The tests compare the two builds bit for bit.
template <int VM>
__device__ __forceinline__ void barrier_keep_vm() {
  static_assert(VM >= 0 && VM < 64, "vmcnt is 6 bits");
#ifdef LASNET_DRAIN_AT_BARRIERS
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#else
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(VM) : "memory");
#endif
}

// The same with a count that is a constant only after unrolling (folds to one of the cases).
template <int I = 63>
__device__ __forceinline__ void barrier_keep_vm_n(int n) {
  if (n >= I) barrier_keep_vm<I>();
  else if constexpr (I > 0) barrier_keep_vm_n<I - 1>(n);
}

// conv1's stream of global-memory operations per wave, in program order (they complete in
// order), for a weight ring of WD chunks and XD chunks of x requested ahead:
//   prologue   c = 0, 1, ..:  W(c) if c < WD,  X(c) if c < XD
//   chunk ch   (barrier, matrix work, and between the MFMAs)  W(ch + WD),  then  X(ch + XD)
// (with the ring filled ahead of the phase -- HOISTED -- the prologue is W(0..WD-1) and then X(0..XD-1)).
// W(c) = the NWL weight fragments of chunk c, X(c) = the NXL x loads of chunk c.  The barrier
// that opens chunk ch needs W(ch) and X(ch) complete; this is the number of operations issued
// after the younger of the two, which may stay in flight.
constexpr int conv1_keep_in_flight(int ch, int nch, int wd, int xd, int nwl, int nxl, bool w_first = false) {
  int after_w = -1, after_x = -1;          // operations issued up to and including W(ch) / X(ch)
  int total = 0;
  auto issue = [&](bool is_w, int c, int n) {
    if (c >= nch) return;
    total += n;
    if (c == ch) { if (is_w) after_w = total; else after_x = total; }
  };
  if (w_first) {                           // the ring was filled before the phase: all of W(0..wd-1), then the x chunks
    for (int c = 0; c < wd; ++c) issue(true, c, nwl);
    for (int c = 0; c < xd; ++c) issue(false, c, nxl);
  } else {
    for (int c = 0; c < (wd > xd ? wd : xd); ++c) {
      if (c < wd) issue(true, c, nwl);
      if (c < xd) issue(false, c, nxl);
    }
  }
  for (int c = 0; c < ch; ++c) { issue(true, c + wd, nwl); issue(false, c + xd, nxl); }
  const int last = after_w > after_x ? after_w : after_x;
  return total - last;
}

// A lane's 4*NB consecutive channels leave as 16-byte pieces (8 channels = one swizzle chunk).
__device__ __forceinline__ bf16x8 join8(bf16x4 a, bf16x4 b) {
  return bf16x8{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
}


// A wave-uniform global pointer that arrived in vector registers (function arguments do)
// -> scalar registers, so that loads through it can take the "scalar base + 32-bit lane
// offset" form: stepping through the weight stream then costs scalar adds only, and no
// vector register pair per load address.
__device__ __forceinline__ g_bf16_p uni_ptr(g_bf16_p p) {
  const unsigned long long v = (unsigned long long)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (g_bf16_p)(((unsigned long long)hi << 32) | lo);
}

// Weights are read with buffer loads: the address is a buffer descriptor (4 scalar registers,
// once per tensor) + a scalar byte offset (the position in the weight stream, wave-uniform)
// + one vector register holding lane * 16 + a 12-bit immediate.  No vector register pair
// and no vector adds per load address, which is what kept the phases from fitting the
// register file when they are inlined into the kernel.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(g_bf16_p p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)(unsigned long long)uni_ptr(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ bf16x8 buf_load16(rsrc_t r, int lane_bytes, int uniform_bytes) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, lane_bytes, uniform_bytes, 0));
}

// ---- phase 1: conv1 over the NB1*16 rows of unique window pixels -------------------------
// x reaches LDS by direct global->LDS loads (16 bytes per lane, a wave fills 8 rows x 128 B;
// the lane picks the global chunk whose swizzled position it writes), three stages deep;
// the weights of the next two chunks are always in flight in registers.
// The weight ring of conv1: WD chunks of KS k-steps, NBW1 fragments each.
template <class K>
struct Conv1Ring { bf16x8 w[K::WD * (K::KC / 32)][K::NBW1]; };
// Requests chunks 0 .. WD-1 (a kernel that has other latencies to wait for does this first).
template <class K>
__device__ __forceinline__ void conv1_ring_fill(Conv1Ring<K>& ring, g_bf16_p W1, int tid, int wave) {
  const rsrc_t wrs = make_rsrc(W1, K::W1_BYTES);
  const int lane16 = (tid & 63) * 16, wbase = (uni(wave) % K::WC1) * K::NBW1 * 1024;
#pragma unroll
  for (int t = 0; t < K::WD * (K::KC / 32); ++t)
#pragma unroll
    for (int j = 0; j < K::NBW1; ++j)
      ring.w[t][j] = buf_load16(wrs, lane16 + j * 1024, wbase + t * K::W_KSTEP_BYTES);
}

// What conv1 runs between requesting its first chunks and waiting for them, when the caller has nothing to put there.
struct Nothing { __device__ __forceinline__ void operator()() const {} };

// HOISTED: `ring` arrives filled by conv1_ring_fill.  yg / nrows: with K::Y1_TO_GLOBAL the result rows
// go straight to memory, row r < nrows to yg + rowpix[r] * K::YG_PITCH (+ channel).  `meanwhile` runs after
// the first chunks of x and weights have been requested and before the first of them is waited for: work
// that needs no global memory hides behind that latency (it must not touch xs or y1s).
template <class K, int NB1, bool HOISTED, class Meanwhile = Nothing>
__device__ LASNET_PHASE_INLINE void conv1_core(Conv1Ring<K>& ring, g_bf16_p x, g_bf16_p W1, l_f32_cp b1s,
                                               l_i32_cp rowpix, l_bf16_p xs, l_bf16_p y1s, int tid, int wave,
                                               AS_GLOBAL __bf16* yg = nullptr, int nrows = 0,
                                               Meanwhile meanwhile = Meanwhile{}) {
  constexpr int C = K::C, NBW = K::NBW1, KS = K::KC / 32, NCH = C / K::KC;
  constexpr int RB = cdiv(NB1, K::WR1);                   // row blocks of this wave (last may be padding)
  constexpr int NGRP = NB1 * 2, NXL = cdiv(NGRP, K::NW);  // 8-row groups; x loads per wave per chunk
  constexpr int NWL = KS * NBW;                           // weight loads per wave per chunk
  const int lane = tid & 63, l16 = lane & 15, lg = lane >> 4;
  const int lane16 = lane * 16;
  wave = uni(wave);
  const int wr = wave / K::WC1, wc = wave % K::WC1;

  // the accumulators start at the bias (read from LDS: the first MFMA of each takes it as its
  // C operand), so the epilogue has no add
  const int chb = wc * NBW * 16;
  floatx4 acc[RB][NBW];
#pragma unroll
  for (int j = 0; j < NBW; ++j) {
    const floatx4 bias = *reinterpret_cast<const AS_LDS floatx4*>(b1s + lane_channel(chb, NBW, j, lg, 0));
#pragma unroll
    for (int i = 0; i < RB; ++i) acc[i][j] = bias;
  }

  // x stream: group u of this wave = rows grp*8 .. grp*8+7
  g_bf16_p xsrc[NXL];
  int xdst[NXL];                                          // element offset inside a stage (wave-uniform)
#pragma unroll
  for (int u = 0; u < NXL; ++u) {
    const int grp = wave + u * K::NW;
    if (grp < NGRP) {
      const int row = grp * 8 + (lane >> 3), pc = lane & 7;
      xsrc[u] = x + (size_t)rowpix[row] * C + ((pc ^ (row & 7)) << 3);
      xdst[u] = grp * 8 * K::LDX;
    } else {                                              // padding load: keeps the per-chunk count uniform
      xsrc[u] = x + (size_t)rowpix[0] * C + ((lane & 7) << 3);
      xdst[u] = K::NSTG * K::STAGE_ELEMS;
    }
  }
  // Direct global->LDS load as inline asm: the compiler must not know that it writes LDS,
  // or it makes every LDS read that follows wait for ALL outstanding global-memory
  // operations (it cannot prove the stages disjoint) and the stream stops being a stream.
  // Completion is tracked by hand instead: see the barrier in the chunk loop.  (m0, which carries
  // the LDS address, is a reserved register: the compiler never keeps a value in it across statements.)
  auto issue_x = [&](int ch) {
    const int stage = ch % K::NSTG;
#pragma unroll
    for (int u = 0; u < NXL; ++u) {
      const int off = xdst[u] == K::NSTG * K::STAGE_ELEMS ? xdst[u] : stage * K::STAGE_ELEMS + xdst[u];
      const unsigned lds_addr = uni((int)(unsigned)(size_t)(xs + off));
      g_bf16_p src = xsrc[u] + ch * K::KC;
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr)
                   : "memory");
    }
  };
  // weights: ring of WD chunks, refilled in place
  constexpr int WD = K::WD;
  const rsrc_t wrs = make_rsrc(W1, K::W1_BYTES);
  const int wbase = (wc * NBW) * 1024;                     // bytes, wave-uniform
  auto& w = ring.w;
  auto wload = [&](int slot, int kstep) {
#pragma unroll
    for (int j = 0; j < NBW; ++j)
      w[slot][j] = buf_load16(wrs, lane16 + j * 1024, wbase + kstep * K::W_KSTEP_BYTES);
  };
  int boff[RB][KS];                                       // LDS offsets of this lane's B fragments
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    const int row = (wr + K::WR1 * i) * 16 + l16;
#pragma unroll
    for (int s = 0; s < KS; ++s) boff[i][s] = swz(row, K::LDX, s * 4 + lg, row, K::XMASK);
  }

  // prologue of the stream (see conv1_keep_in_flight for the order)
  constexpr int XD = K::XD;
#pragma unroll
  for (int c = 0; c < (WD > XD ? WD : XD); ++c) {
    if (!HOISTED && c < WD && c < NCH) {
#pragma unroll
      for (int t = 0; t < KS; ++t) wload(c * KS + t, c * KS + t);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (c < XD) {
      issue_x(c);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  meanwhile();
  __builtin_amdgcn_sched_barrier(0);

  // B fragments are read one k-step ahead of the MFMAs that use them (bcur/bnxt), so a
  // wave's LDS latency hides behind its own matrix work.
  bf16x8 bcur[RB], bnxt[RB];
  // fully unrolled: with a back edge the compiler's own waits for the weight registers fall
  // back to vmcnt(0), which would drain the x stream every other chunk
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    {
      const int cc = ch % WD;                              // ring slot group of this chunk (constant after unrolling)
      barrier_keep_vm_n(conv1_keep_in_flight(ch, NCH, WD, XD, NWL, NXL, HOISTED));
      __builtin_amdgcn_sched_barrier(0);
      l_bf16_cp xb = xs + (ch % K::NSTG) * K::STAGE_ELEMS;
#pragma unroll
      for (int i = 0; i < RB; ++i) bcur[i] = *reinterpret_cast<const AS_LDS bf16x8*>(xb + boff[i][0]);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        if (s + 1 < KS) {
#pragma unroll
          for (int i = 0; i < RB; ++i) bnxt[i] = *reinterpret_cast<const AS_LDS bf16x8*>(xb + boff[i][s + 1]);
        }
#pragma unroll
        for (int i = 0; i < RB; ++i)
#pragma unroll
          for (int j = 0; j < NBW; ++j) acc[i][j] = mfma16(w[cc * KS + s][j], bcur[i], acc[i][j]);
        if (ch + WD < NCH) wload(cc * KS + s, (ch + WD) * KS + s);
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < KS) {
#pragma unroll
          for (int i = 0; i < RB; ++i) bcur[i] = bnxt[i];
        }
      }
      // the stage of chunk ch+XD was last read during chunk ch-1, which every wave has left
      // (barrier above)
      if (ch + XD < NCH) issue_x(ch + XD);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // (y1s may lie inside the x stages: every wave must have read its last chunk first)
  if constexpr (K::Y1_IN_XS) __syncthreads();
  // epilogue: ReLU, round to bf16; 8 channels (one 16-byte chunk) per LDS store where NBW allows
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    const int row = (wr + K::WR1 * i) * 16 + l16;
    bf16x4 o[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) o[j][v] = (__bf16)fmaxf(acc[i][j][v], 0.f);
    if constexpr (K::Y1_TO_GLOBAL) {
      static_assert(!K::Y1_TO_GLOBAL || NBW % 2 == 0, "16-byte pieces");
      if (row < nrows) {
        AS_GLOBAL __bf16* dst = yg + (size_t)rowpix[row] * K::YG_PITCH;
#pragma unroll
        for (int j = 0; j < NBW; j += 2)
          *reinterpret_cast<AS_GLOBAL bf16x8*>(dst + lane_channel(chb, NBW, j, lg, 0)) = join8(o[j], o[j + 1]);
      }
    } else if constexpr (NBW % 2 == 0) {
#pragma unroll
      for (int j = 0; j < NBW; j += 2)
        *reinterpret_cast<AS_LDS bf16x8*>(y1s + swz(row, K::LDY, lane_channel(chb, NBW, j, lg, 0) >> 3, row, K::YMASK)) = join8(o[j], o[j + 1]);
    } else {
#pragma unroll
      for (int j = 0; j < NBW; ++j) {
        const int c = lane_channel(chb, NBW, j, lg, 0);
        *reinterpret_cast<AS_LDS bf16x4*>(y1s + swz(row, K::LDY, c >> 3, row, K::YMASK) + (c & 7)) = o[j];
      }
    }
  }
}

template <class K, int NB1, class Meanwhile = Nothing>
__device__ LASNET_PHASE_INLINE void conv1_phase(g_bf16_p x, g_bf16_p W1, l_f32_cp b1s, l_i32_cp rowpix,
                                                l_bf16_p xs, l_bf16_p y1s, int tid, int wave,
                                                Meanwhile meanwhile = Meanwhile{}) {
  Conv1Ring<K> ring;
  conv1_core<K, NB1, false>(ring, x, W1, b1s, rowpix, xs, y1s, tid, wave, nullptr, 0, meanwhile);
}

// ---- phase 2: conv3x3 as an implicit GEMM over the 9 taps, y1 rows from LDS ---------------
// The weight ring of conv2: the next RD2 k-steps, NBW2 fragments each.
template <class K>
struct Conv2Ring { bf16x8 w[K::RD2][K::NBW2]; };
template <class K>
__device__ __forceinline__ void conv2_ring_fill(Conv2Ring<K>& ring, g_bf16_p W2, int tid, int wave) {
  const rsrc_t wrs = make_rsrc(W2, K::W2_BYTES);
  const int lane16 = (tid & 63) * 16, wbase = (uni(wave) % K::WC2) * K::NBW2 * 1024;
#pragma unroll
  for (int t = 0; t < K::RD2; ++t)
#pragma unroll
    for (int j = 0; j < K::NBW2; ++j)
      ring.w[t][j] = buf_load16(wrs, lane16 + j * 1024, wbase + t * K::W_KSTEP_BYTES);
}

// HOISTED: `ring` arrives holding k-steps 0 .. RD-1 and is left holding them again (the refills wrap
// around), ready for another pass.  yg: with K::Y2_TO_GLOBAL the result rows go straight to memory,
// row q < nq to yg + q * K::YG_PITCH (+ channel).
template <class K, int NB2, bool HOISTED>
__device__ LASNET_PHASE_INLINE void conv2_core(Conv2Ring<K>& ring, g_bf16_p W2, l_f32_cp b2s, l_i16_cp winrow,
                                               l_bf16_cp y1s, l_bf16_p y2s, int nq, int tid, int wave,
                                               AS_GLOBAL __bf16* yg = nullptr) {
  constexpr int S = K::S, T = K::T, WW = K::WW;
  constexpr int NBW = K::NBW2, MS = K::MS, RD = K::RD2, NSTEP = 9 * MS;
  constexpr int RB = cdiv(NB2, K::WR2);
  const int lane = tid & 63, l16 = lane & 15, lg = lane >> 4;
  const int lane16 = lane * 16;
  wave = uni(wave);
  const int wr = wave / K::WC2, wc = wave % K::WC2;
  const int chb = wc * NBW * 16;
  floatx4 acc[RB][NBW];                                    // start at the bias, like conv1's
#pragma unroll
  for (int j = 0; j < NBW; ++j) {
    const floatx4 bias = *reinterpret_cast<const AS_LDS floatx4*>(b2s + lane_channel(chb, NBW, j, lg, 0));
#pragma unroll
    for (int i = 0; i < RB; ++i) acc[i][j] = bias;
  }
  int wpos[RB];                                            // window position of tap (0,0)
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    const int q = (wr + K::WR2 * i) * 16 + l16;
    wpos[i] = -1;
    if (q < nq) {
      const int slot = q / (S * S), r = q - slot * (S * S);
      wpos[i] = slot * WW + (r / S) * T + r % S;
    }
  }
  const rsrc_t wrs = make_rsrc(W2, K::W2_BYTES);
  const int wbase = (wc * NBW) * 1024;                     // bytes, wave-uniform
  auto& w = ring.w;                                        // weights of the next RD k-steps, refilled in place
  auto wload = [&](int slot, int kstep) {
#pragma unroll
    for (int j = 0; j < NBW; ++j)
      w[slot][j] = buf_load16(wrs, lane16 + j * 1024, wbase + kstep * K::W_KSTEP_BYTES);
  };
  if constexpr (!HOISTED) {
#pragma unroll
    for (int t = 0; t < RD; ++t) wload(t, t);
  }
  // The caller may have left the direct global->LDS loads of y1 in flight and the row tables unsynchronised:
  // everything this wave has requested so far must have landed, and every wave must have got here.
  if constexpr (K::ACTS_BARRIER) {
    __builtin_amdgcn_sched_barrier(0);
    barrier_keep_vm<HOISTED ? 0 : RD * NBW>();
    __builtin_amdgcn_sched_barrier(0);
  }
  auto lookup = [&](int (&br)[RB], int tap) {
    const int toff = (tap / 3) * T + tap % 3;
#pragma unroll
    for (int i = 0; i < RB; ++i) br[i] = wpos[i] >= 0 ? winrow[wpos[i] + toff] : K::ZROW;
  };
  int brow[RB];
  FragRow fr[RB];
  lookup(brow, 0);
#pragma unroll
  for (int i = 0; i < RB; ++i) fr[i] = frag_row(brow[i], K::LDY, lg, brow[i], K::YMASK);
  // B fragments one k-step ahead of the MFMAs (bcur/bnxt); the row lookup of the next tap
  // happens while the last k-step of the current one is computed.
  bf16x8 bcur[RB], bnxt[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i) bcur[i] = frag_read(y1s, fr[i], 0);
  // fully unrolled (as in conv1): across a back edge the compiler's waits for the weight ring
  // degrade towards vmcnt(0) and the ring stops hiding any latency
#pragma unroll
  for (int t0 = 0; t0 < NSTEP; t0 += RD) {
#pragma unroll
    for (int tt = 0; tt < RD; ++tt) {
      const int t = t0 + tt;
      const int msn = (t + 1) % MS;                        // k-step inside the tap of step t+1
      if (t + 1 < NSTEP) {
        if (msn == 0) {
          lookup(brow, (t + 1) / MS);
#pragma unroll
          for (int i = 0; i < RB; ++i) fr[i] = frag_row(brow[i], K::LDY, lg, brow[i], K::YMASK);
        }
#pragma unroll
        for (int i = 0; i < RB; ++i) bnxt[i] = frag_read(y1s, fr[i], msn);
      }
#pragma unroll
      for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int j = 0; j < NBW; ++j) acc[i][j] = mfma16(w[tt][j], bcur[i], acc[i][j]);
      if (HOISTED || t + RD < NSTEP) wload(tt, (t + RD) % NSTEP);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < RB; ++i) bcur[i] = bnxt[i];
    }
  }
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    const int q = (wr + K::WR2 * i) * 16 + l16;
    bf16x4 o[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) o[j][v] = (__bf16)fmaxf(acc[i][j][v], 0.f);
    if constexpr (K::Y2_TO_GLOBAL) {
      static_assert(!K::Y2_TO_GLOBAL || NBW % 2 == 0, "16-byte pieces");
      if (q < nq) {
#pragma unroll
        for (int j = 0; j < NBW; j += 2)
          *reinterpret_cast<AS_GLOBAL bf16x8*>(yg + (size_t)q * K::YG_PITCH + lane_channel(chb, NBW, j, lg, 0)) = join8(o[j], o[j + 1]);
      }
    } else if constexpr (NBW % 2 == 0) {
#pragma unroll
      for (int j = 0; j < NBW; j += 2)
        *reinterpret_cast<AS_LDS bf16x8*>(y2s + swz(q, K::LDY2, lane_channel(chb, NBW, j, lg, 0) >> 3, q, K::YMASK2)) = join8(o[j], o[j + 1]);
    } else {
#pragma unroll
      for (int j = 0; j < NBW; ++j) {
        const int c = lane_channel(chb, NBW, j, lg, 0);
        *reinterpret_cast<AS_LDS bf16x4*>(y2s + swz(q, K::LDY2, c >> 3, q, K::YMASK2) + (c & 7)) = o[j];
      }
    }
  }
}

// ---- phase 3: conv3 + b3 + residual, one rounding, stored at the patch's own pixels -------
// The weight ring of conv3: the next RD3 k-steps of NB3 fragments; a wave's stream is contiguous over
// (pass, k-step, tile).  wc0: wave columns that other workgroups take (output channels split across workgroups).
template <class K>
struct Conv3Ring { bf16x8 w[K::RD3][K::NB3]; };
template <class K>
__device__ __forceinline__ void conv3_ring_fill(Conv3Ring<K>& ring, g_bf16_p W3, int tid, int wave, int wc0 = 0) {
  const rsrc_t wrs = make_rsrc(W3, K::W3_BYTES);
  const int lane16 = (tid & 63) * 16;
  const int wbase = ((wc0 + uni(wave) % K::WC3) * (K::NBT3 / K::NB3)) * K::MS * K::NB3 * 1024;
#pragma unroll
  for (int t = 0; t < K::RD3; ++t)
#pragma unroll
    for (int j = 0; j < K::NB3; ++j)
      ring.w[t][j] = buf_load16(wrs, lane16 + j * 1024, wbase + t * (K::NB3 * 1024));
}

// The residual (x at the output pixels) of conv3's first pass, in the registers of the lanes that will add it.
template <class K, int NB2>
struct Conv3Residual { bf16x8 v[cdiv(NB2, K::WR3)][K::NB3 / 2]; };
// Requests it.  The fused kernel does this at the start of conv2, a phase that reads no global memory but
// its weights: the loads have landed long before conv3 starts (which otherwise opens with this wait), and
// they run while the memory system is idle instead of beside conv3's stores.
template <class K, int NB2>
__device__ __forceinline__ void conv3_residual_request(Conv3Residual<K, NB2>& res, g_bf16_p x, l_i32_cp pixq,
                                                       int tid, int wave, int wc0 = 0) {
  const int lane = tid & 63, l16 = lane & 15, lg = lane >> 4;
  wave = uni(wave);
  const int wr = wave / K::WC3, wc = wc0 + wave % K::WC3;
  const int chb = (wc * K::NBT3) * 16;
#pragma unroll
  for (int i = 0; i < cdiv(NB2, K::WR3); ++i) {
    const int pq = pixq[(wr + K::WR3 * i) * 16 + l16];     // rows past the last pixel read pixel 0 (never stored)
#pragma unroll
    for (int j = 0; j < K::NB3 / 2; ++j)
      res.v[i][j] = *reinterpret_cast<const AS_GLOBAL bf16x8*>(x + (size_t)max(pq, 0) * K::C + lane_channel(chb, K::NB3, 2 * j, lg, 0));
  }
}

// HOISTED: `ring` arrives holding steps 0 .. RD-1 and is left holding them again (the refills wrap around).
// res0: the first pass's residual if the caller has requested it already (conv3_residual_request), else null.
template <class K, int NB2, bool HOISTED>
__device__ LASNET_PHASE_INLINE void conv3_core(Conv3Ring<K>& ring, g_bf16_p x, g_bf16_p W3, l_f32_cp b3s,
                                               l_i32_cp pixq, l_bf16_cp y2s, l_bf16_p tscratch,
                                               AS_GLOBAL __bf16* out, int post_relu, int tid, int wave, int wc0 = 0,
                                               const Conv3Residual<K, NB2>* res0 = nullptr) {
  constexpr int C = K::C, NB = K::NB3, MS = K::MS, RD = K::RD3;
  constexpr int NPASS = K::NBT3 / NB, NSTEP = NPASS * MS;
  constexpr int RB = cdiv(NB2, K::WR3);
  const int lane = tid & 63, l16 = lane & 15, lg = lane >> 4;
  const int lane16 = lane * 16;
  wave = uni(wave);
  // wc0: wave columns that other workgroups take (when the output channels are split across workgroups)
  const int wr = wave / K::WC3, wc = wc0 + wave % K::WC3;
  const float floor_ = post_relu ? 0.f : -__builtin_inff();   // ReLU after the add, or nothing
  int pq[RB];
  FragRow fr[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    const int bq = (wr + K::WR3 * i) * 16 + l16;
    fr[i] = frag_row(bq, K::LDY, lg, bq, K::YMASK);
  }
  // this wave's weight stream is contiguous over (pass, k-step, tile)
  const rsrc_t wrs = make_rsrc(W3, K::W3_BYTES);
  const int wbase = (wc * NPASS) * MS * NB * 1024;         // bytes, wave-uniform
  auto& w = ring.w;
  auto wload = [&](int slot, int t) {
#pragma unroll
    for (int j = 0; j < NB; ++j)
      w[slot][j] = buf_load16(wrs, lane16 + j * 1024, wbase + t * (NB * 1024));
  };
  if constexpr (!HOISTED) {
#pragma unroll
    for (int t = 0; t < RD; ++t) wload(t, t);
  }
  if constexpr (K::ACTS_BARRIER) {                         // as in conv2: y2 rows requested by the caller, pixq unsynchronised
    __builtin_amdgcn_sched_barrier(0);
    barrier_keep_vm<HOISTED ? 0 : RD * NB>();
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int i = 0; i < RB; ++i) pq[i] = pixq[(wr + K::WR3 * i) * 16 + l16];
  // The residual comes from HBM, the weights from L2, and a wave's loads complete in issue order:
  // a weight fragment requested after a residual load cannot be used before that load has landed.
  // So a pass's residual is requested as early as its registers allow, straight after the weights
  // that are already due: for pass 0 here, for pass p+1 between the GEMM and the epilogue of pass p
  // (the epilogue and the ring's depth then cover its latency).
  bf16x8 xres[2][RB][NB / 2];
  auto rload = [&](int pass) {
    const int chb = (wc * K::NBT3 + pass * NB) * 16;
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int j = 0; j < NB / 2; ++j)   // rows past the last pixel read pixel 0 (never stored)
        xres[pass & 1][i][j] = *reinterpret_cast<const AS_GLOBAL bf16x8*>(x + (size_t)max(pq[i], 0) * C + lane_channel(chb, NB, 2 * j, lg, 0));
  };
  if (res0) {
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int j = 0; j < NB / 2; ++j) xres[0][i][j] = res0->v[i][j];
  } else {
    rload(0);
  }
  // fully unrolled, like conv1 and conv2: the weight ring runs on across the passes
#pragma unroll
  for (int pass = 0; pass < NPASS; ++pass) {
    const int chb = (wc * K::NBT3 + pass * NB) * 16;       // first channel of this wave's pass
    floatx4 acc[RB][NB];                                   // start at the bias
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const floatx4 bias = *reinterpret_cast<const AS_LDS floatx4*>(b3s + lane_channel(chb, NB, j, lg, 0));
#pragma unroll
      for (int i = 0; i < RB; ++i) acc[i][j] = bias;
    }
    bf16x8 bcur[RB], bnxt[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) bcur[i] = frag_read(y2s, fr[i], 0);
#pragma unroll
    for (int s = 0; s < MS; ++s) {
      if (s + 1 < MS) {
#pragma unroll
        for (int i = 0; i < RB; ++i) bnxt[i] = frag_read(y2s, fr[i], s + 1);
      }
#pragma unroll
      for (int i = 0; i < RB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = mfma16(w[s % RD][j], bcur[i], acc[i][j]);
      // refill with the step RD ahead (the stream runs on into the next pass; past its end the
      // last step is re-read, unused)
      wload(s % RD, HOISTED ? (pass * MS + s + RD) % NSTEP : min(pass * MS + s + RD, NSTEP - 1));
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < MS) {
#pragma unroll
        for (int i = 0; i < RB; ++i) bcur[i] = bnxt[i];
      }
    }
    if (pass + 1 < NPASS) rload(pass + 1);
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      bf16x8 o[NB / 2];
#pragma unroll
      for (int j = 0; j < NB; j += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            o[j / 2][h * 4 + v] = (__bf16)fmaxf((float)xres[pass & 1][i][j / 2][h * 4 + v] + acc[i][j + h][v], floor_);
          }
        }
      }
      // Streaming stores (out is not read again here; lines left dirty in L2 would all be written
      // back in one burst when the kernel ends).
      if constexpr (NB == 4) {
        // A pass gives a lane 2 x 16 bytes of its pixel and the four lane groups one 128-byte line of
        // it, but a store instruction in that layout scatters 16-byte pieces over 16 lines.  The
        // wave transposes the 16 x 128 bytes through 2 KiB of LDS of its own (inside the y1 region,
        // which is dead during conv3; rows swizzled like every other LDS row), so that each store
        // instruction writes 8 whole lines, 8 consecutive lanes per line.
        AS_LDS char* tr = reinterpret_cast<AS_LDS char*>(tscratch) + wave * 2048;
#pragma unroll
        for (int t = 0; t < 2; ++t)
          *reinterpret_cast<AS_LDS bf16x8*>(tr + l16 * 128 + (((4 * t + lg) ^ (l16 & 7)) << 4)) = o[t];
        const int c8 = lane & 7;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int p = half * 8 + (lane >> 3);                    // pixel (row of the block) this lane stores for
          const bf16x8 v = *reinterpret_cast<const AS_LDS bf16x8*>(tr + p * 128 + ((c8 ^ (p & 7)) << 4));
          const int pix = pixq[(wr + K::WR3 * i) * 16 + p];
          if (pix >= 0)
            __builtin_nontemporal_store(v, reinterpret_cast<AS_GLOBAL bf16x8*>(out + (size_t)pix * C + chb + c8 * 8));
        }
      } else {
        if (pq[i] >= 0) {
#pragma unroll
          for (int j = 0; j < NB; j += 2)
            __builtin_nontemporal_store(o[j / 2], reinterpret_cast<AS_GLOBAL bf16x8*>(
                                                      out + (size_t)pq[i] * C + lane_channel(chb, NB, j, lg, 0)));
        }
      }
    }
  }
}

template <class K>
__global__ __launch_bounds__(K::NT, K::WAVES_PER_SIMD) void fused_bneck_kernel(
    Geom g, int tile_slots, const __bf16* __restrict__ x, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ count, const __bf16* __restrict__ W1,
    const float* __restrict__ b1, const __bf16* __restrict__ W2, const float* __restrict__ b2,
    const __bf16* __restrict__ W3, const float* __restrict__ b3, __bf16* __restrict__ out,
    int post_relu) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int* hkey = reinterpret_cast<int*>(smem + K::OFF_HKEY);
  short* hval = reinterpret_cast<short*>(smem + K::OFF_HVAL);
  short* winrow = reinterpret_cast<short*>(smem + K::OFF_WINROW);
  int* rowpix = reinterpret_cast<int*>(smem + K::OFF_ROWPIX);
  int* pixq = reinterpret_cast<int*>(smem + K::OFF_PIXQ);
  int* misc = reinterpret_cast<int*>(smem + K::OFF_MISC);      // [0] = number of unique rows
  int* cellq = reinterpret_cast<int*>(smem + K::OFF_CELL);
  float* b1s = reinterpret_cast<float*>(smem + K::OFF_BIAS);
  float* b2s = b1s + K::M;
  float* b3s = b2s + K::M;
  __bf16* y1s = reinterpret_cast<__bf16*>(smem + K::OFF_Y1);
  __bf16* xs = reinterpret_cast<__bf16*>(smem + K::OFF_XS);
  __bf16* y2s = xs;                                        // xs is dead once conv1 is done

  constexpr int S = K::S, T = K::T, WW = K::WW;
  const int tid = threadIdx.x;
  const int wave = uni(tid >> 6);

  // ---- which entries of the index list are this workgroup's ------------------------------
  // The list is cut into `nt` near-equal runs, nt = the number of PPW-sized tiles rounded up
  // to a multiple of `tile_slots` (workgroups the chip holds at once), so that every round
  // of workgroups is full whatever the count turns out to be.
  const int nact = uni(idx ? min(*count, g.P) : g.P);
  if (nact <= 0) return;
  int nt = (nact + K::PPW - 1) / K::PPW;
  nt = (nt + tile_slots - 1) / tile_slots * tile_slots;
  nt = min(min(nt, (int)gridDim.x), nact);
  if ((int)blockIdx.x >= nt) return;                       // uniform over the workgroup
  // Workgroup b runs on XCD b % 8 (round-robin dispatch), and each XCD has its own L2.  Runs
  // that are neighbours in the list share window pixels, so XCD k takes a contiguous eighth
  // of the runs: the shared rows are then fetched into one L2 once, not into two.
  // Within its eighth, an XCD's longer runs (one entry more than the others) go to its FIRST workgroups:
  // when the launch takes more than one round of workgroups, a run that needs a second batch (a
  // batch is cut when its windows share too little) then starts early instead of ending the launch.
  const int xcd = (int)blockIdx.x & 7, jx = (int)blockIdx.x >> 3;
  const int first = xcd * (nt >> 3) + min(xcd, nt & 7);        // jx < runs of this XCD because b < nt
  const int runs = (nt >> 3) + (xcd < (nt & 7) ? 1 : 0);
  const int xb = (int)(((long long)first * nact) / nt), xe = (int)(((long long)(first + runs) * nact) / nt);
  const int len0 = (xe - xb) / runs, extra = (xe - xb) - len0 * runs;
  const int tb = xb + jx * len0 + min(jx, extra);
  const int te = tb + len0 + (jx < extra ? 1 : 0);

  // the all-zero y1 row
  for (int i = tid; i < K::LDY / 8; i += K::NT)
    *reinterpret_cast<uint4*>(y1s + K::ZROW * K::LDY + i * 8) = uint4{0, 0, 0, 0};
  // the biases go to LDS: requested here, stored once the first batch's cell ids (requested next)
  // have been waited for anyway
  constexpr int NBV = cdiv(2 * K::M + K::C, K::NT);
  float bv[NBV];
#pragma unroll
  for (int u = 0; u < NBV; ++u) {
    const int i = tid + u * K::NT;
    bv[u] = i < K::M ? b1[i] : i < 2 * K::M ? b2[i - K::M] : i < 2 * K::M + K::C ? b3[i - 2 * K::M] : 0.f;
  }

  for (int e0 = tb; e0 < te;) {
    // ---------------------------------------------------------------- phase 0
    int npb = min(te - e0, K::PPW);                        // patches in this batch
    int U;                                                 // unique window pixels = y1 rows
    // the batch's cell ids: one round of global loads, every later step reads them from LDS
    for (int i = tid; i < npb; i += K::NT) cellq[i] = idx ? idx[e0 + i] : e0 + i;
    if (e0 == tb) {
#pragma unroll
      for (int u = 0; u < NBV; ++u)
        if (tid + u * K::NT < 2 * K::M + K::C) b1s[tid + u * K::NT] = bv[u];   // b1 | b2 | b3 are contiguous
    }
    for (;;) {
      for (int i = tid; i < K::HT; i += K::NT) hkey[i] = 0;
      if (tid == 0) misc[0] = 0;
      __syncthreads();
      // (a) every in-image window pixel claims a hash slot
      for (int t = tid; t < npb * WW; t += K::NT) {
        const int slot = t / WW, wp = t - slot * WW;
        const int cell = cellq[slot];
        const int n = cell / (g.G * g.GW), rem = cell - n * (g.G * g.GW);
        const int gy = rem / g.GW, gx = rem - gy * g.GW;
        const int h = gy * S + wp / T - 1, w = gx * S + wp % T - 1;
        // (a list entry that is not a cell of this map claims nothing and stores nothing)
        if ((unsigned)cell < (unsigned)g.P && h >= 0 && h < g.H && w >= 0 && w < g.W) {
          const int key = (n * g.H + h) * g.W + w + 1;
          unsigned s = hash_pix(key) & (K::HT - 1);
          for (;;) {
            const int old = atomicCAS(&hkey[s], 0, key);
            if (old == 0 || old == key) break;
            s = (s + 1) & (K::HT - 1);
          }
        }
      }
      __syncthreads();
      // (b) occupied slots take row numbers
      for (int i = tid; i < K::HT; i += K::NT) {
        const int key = hkey[i];
        if (key != 0) {
          const int row = atomicAdd(&misc[0], 1);
          hval[i] = (short)row;
          if (row < K::R1MAX) rowpix[row] = key - 1;
        }
      }
      __syncthreads();
      U = uni(misc[0]);
      if (U <= K::R1MAX) break;
      // too many distinct pixels for the y1 buffer: retry with fewer patches (WW <= R1MAX, so
      // one patch always fits)
      npb = max(1, min(npb - 1, npb * K::R1MAX / U));
      __syncthreads();
    }
    const int nblk1 = max(1, (U + 15) >> 4);              // (U = 0 only if every entry of the batch was invalid)
    const int nq = npb * S * S, nblk2 = (nq + 15) >> 4;
    // rows up to the block count conv1 really runs (rounded up to its wave rows) must name
    // a valid pixel: their x is loaded and convolved, the result is never used
    const int pad_pix = U > 0 ? rowpix[0] : 0;
    for (int r = U + tid; r < (nblk1 + K::WR1 - 1) / K::WR1 * K::WR1 * 16; r += K::NT) rowpix[r] = pad_pix;
    __syncthreads();
    // (c) row of every window position; pixel of every output row.  Only conv2 and conv3 need these, so
    // they are built inside conv1, between the request for its first chunks of x and the wait for them.
    const auto tables = [&] {
      for (int t = tid; t < npb * WW; t += K::NT) {
        const int slot = t / WW, wp = t - slot * WW;
        const int cell = cellq[slot];
        const int n = cell / (g.G * g.GW), rem = cell - n * (g.G * g.GW);
        const int gy = rem / g.GW, gx = rem - gy * g.GW;
        const int h = gy * S + wp / T - 1, w = gx * S + wp % T - 1;
        int row = K::ZROW;
        if ((unsigned)cell < (unsigned)g.P && h >= 0 && h < g.H && w >= 0 && w < g.W) {
          const int key = (n * g.H + h) * g.W + w + 1;
          unsigned s = hash_pix(key) & (K::HT - 1);
          while (hkey[s] != key) s = (s + 1) & (K::HT - 1);
          row = hval[s];
        }
        winrow[t] = (short)row;
      }
      for (int q = tid; q < K::R2P; q += K::NT) {
        int pix = -1;
        if (q < nq) {
          const int slot = q / (S * S), r = q - slot * (S * S);
          const int cell = cellq[slot];
          const int n = cell / (g.G * g.GW), rem = cell - n * (g.G * g.GW);
          const int gy = rem / g.GW, gx = rem - gy * g.GW;
          if ((unsigned)cell < (unsigned)g.P) pix = (n * g.H + gy * S + r / S) * g.W + gx * S + r % S;
        }
        pixq[q] = pix;
      }
    };

    // Row blocks are dealt to the wave rows round-robin (wave row wr takes blocks wr, wr+WR,
    // ...); the count is rounded up to a multiple of WR, the extra blocks compute unused rows.
    dispatch_count<1, K::R1B / K::WR1>((nblk1 + K::WR1 - 1) / K::WR1, [&](auto nb) {
      conv1_phase<K, decltype(nb)::value * K::WR1>((g_bf16_p)x, (g_bf16_p)W1, (l_f32_cp)b1s, (l_i32_cp)rowpix,
                                                   (l_bf16_p)xs, (l_bf16_p)y1s, opaque(tid), wave, tables);
    });
    __syncthreads();
    constexpr int WR23 = K::WR2 > K::WR3 ? K::WR2 : K::WR3;
    // conv2 and conv3 share one dispatch on the block count: conv3's first residual is requested at the
    // start of conv2 and handed over in registers
    dispatch_count<1, K::R2B / WR23>((nblk2 + WR23 - 1) / WR23, [&](auto nb) {
      constexpr int NB2 = decltype(nb)::value * WR23;
      // conv3 keeps a row block's whole output line in registers: it takes the batch's rows in groups of at most
      // NB3ROWS blocks (its weights stream again for the second group; a second batch would stream all three)
      constexpr int NB3A = NB2 < K::NB3ROWS ? NB2 : K::NB3ROWS, NB3B = NB2 - NB3A;
      static_assert(NB3B <= K::NB3ROWS && (NB3B == 0 || (NB3A * 16) % 16 == 0), "two groups of row blocks at most");
      // conv2's first weights are requested before the residual: a wave's loads complete in issue order,
      // and these come from L2 while the residual comes from memory
      Conv2Ring<K> ring2;
      conv2_ring_fill<K>(ring2, (g_bf16_p)W2, opaque(tid), wave);
      Conv3Residual<K, NB3A> res;
      conv3_residual_request<K, NB3A>(res, (g_bf16_p)x, (l_i32_cp)pixq, opaque(tid), wave);
      // (the ring arrives filled; the first k-steps it re-requests at the end are not used)
      conv2_core<K, NB2, true>(ring2, (g_bf16_p)W2, (l_f32_cp)b2s, (l_i16_cp)winrow, (l_bf16_cp)y1s, (l_bf16_p)y2s,
                               nq, opaque(tid), wave);
      __syncthreads();
      Conv3Ring<K> ring3;
      conv3_core<K, NB3A, false>(ring3, (g_bf16_p)x, (g_bf16_p)W3, (l_f32_cp)b3s, (l_i32_cp)pixq, (l_bf16_cp)y2s,
                                 (l_bf16_p)y1s, (AS_GLOBAL __bf16*)out, post_relu, opaque(tid), wave, 0, &res);
      if constexpr (NB3B > 0) {
        // rows NB3A*16 ..: a whole number of swizzle periods further on, so the row keys conv2 wrote them with still fit
        Conv3Ring<K> ring3b;
        conv3_core<K, NB3B, false>(ring3b, (g_bf16_p)x, (g_bf16_p)W3, (l_f32_cp)b3s, (l_i32_cp)pixq + NB3A * 16,
                                   (l_bf16_cp)y2s + NB3A * 16 * K::LDY, (l_bf16_p)y1s, (AS_GLOBAL __bf16*)out, post_relu,
                                   opaque(tid), wave);
      }
    });
    e0 += npb;
    if (e0 < te) __syncthreads();                          // LDS is reused by the next batch
  }
}

// Rewrites W1|W2|W3 in the order the fused kernel's waves consume them: one 16x32 MFMA
// A-fragment (64 lanes x 16 bytes) per contiguous KiB, fragments of one k-step next to
// each other.  A wave's weight stream is then a run of whole cache lines spread over all
// L2 channels, instead of 64-byte pieces of rows that sit a power of two apart (which
// measured 2x slower end to end).
template <class K>
__global__ __launch_bounds__(256) void pack_weights_kernel(const __bf16* __restrict__ W1,
                                                           const __bf16* __restrict__ W2,
                                                           const __bf16* __restrict__ W3,
                                                           __bf16* __restrict__ packed) {
  constexpr int C = K::C, M = K::M, MS = K::MS;
  constexpr int N1 = M * C / 8, N2 = 9 * M * M / 8, N3 = C * M / 8;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= N1 + N2 + N3) return;
  const int lane = t & 63, l16 = lane & 15, lg = lane >> 4;
  const __bf16* src;
  if (t < N1) {
    const int f = t >> 6, kstep = f / (M / 16), fb = f % (M / 16);
    const int wc = fb / K::NBW1, j = fb % K::NBW1;
    src = W1 + (size_t)arow_channel(wc * K::NBW1 * 16, K::NBW1, j, l16) * C + kstep * 32 + 8 * lg;
  } else if (t < N1 + N2) {
    const int f = (t - N1) >> 6, kstep = f / (M / 16), fb = f % (M / 16);
    const int wc = fb / K::NBW2, j = fb % K::NBW2;
    src = W2 + (size_t)arow_channel(wc * K::NBW2 * 16, K::NBW2, j, l16) * (9 * M) + kstep * 32 + 8 * lg;
  } else {
    constexpr int NPASS = K::NBT3 / K::NB3;
    int f = (t - N1 - N2) >> 6;
    const int j = f % K::NB3; f /= K::NB3;
    const int step = f % MS; f /= MS;
    const int pass = f % NPASS, wc = f / NPASS;
    src = W3 + (size_t)arow_channel((wc * K::NBT3 + pass * K::NB3) * 16, K::NB3, j, l16) * M + step * 32 + 8 * lg;
  }
  *reinterpret_cast<uint4*>(packed + (size_t)t * 8) = *reinterpret_cast<const uint4*>(src);
}

template <class K>
hipError_t pack_one(const void* W1, const void* W2, const void* W3, void* packed, hipStream_t st) {
  hipLaunchKernelGGL(pack_weights_kernel<K>, dim3((unsigned)((K::PACKED_ELEMS / 8 + 255) / 256)), dim3(256), 0,
                     st, (const __bf16*)W1, (const __bf16*)W2, (const __bf16*)W3, (__bf16*)packed);
  return hipGetLastError();
}

// A kernel that needs more than 64 KiB of dynamic LDS must be told so once per device.
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = dev < 64 ? 1ull << dev : 0ull;    // devices past 63: set every time
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

template <class K>
hipError_t prepare_one() {
  static std::atomic<unsigned long long> lds_allowed{0};
  return allow_dynamic_lds((const void*)fused_bneck_kernel<K>, K::LDS_BYTES, lds_allowed);
}

template <class K>
hipError_t launch_one(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                      const void* packed, const float* b1, const float* b2, const float* b3,
                      void* out, bool post_relu, hipStream_t st) {
  auto k = fused_bneck_kernel<K>;
  if (hipError_t e = prepare_one<K>(); e != hipSuccess) return e;
  const int slots = device_cu_count() * ((160 * 1024) / K::LDS_BYTES);
  int grid = (g.P + K::PPW - 1) / K::PPW;
  grid = (grid + slots - 1) / slots * slots;
  if (grid > g.P) grid = g.P;
  const __bf16* p1 = (const __bf16*)packed;
  const __bf16* p2 = p1 + (size_t)K::M * K::C;
  const __bf16* p3 = p2 + 9 * (size_t)K::M * K::M;
  hipLaunchKernelGGL(k, dim3(grid), dim3(K::NT), K::LDS_BYTES, st, g, slots, (const __bf16*)x, idx,
                     count, p1, b1, p2, b2, p3, b3, (__bf16*)out, (int)post_relu);
  return hipGetLastError();
}


template <class K>
constexpr MfmaVariant variant_of() {
  return MfmaVariant{K::C, K::M, K::S, K::PACKED_ELEMS * 2, 0, &prepare_one<K>, &pack_one<K>, &launch_one<K>};
}

}  // namespace

// A translation unit lists its instantiations with X-macros and exports them as one table.
#define LASNET_VARIANT_ENTRY(K) variant_of<K>(),
#define LASNET_DEFINE_VARIANT_TABLE(name, CFGS)                     \
  const MfmaVariant* mfma_variants_##name(int* n) {                 \
    static const MfmaVariant table[] = {CFGS(LASNET_VARIANT_ENTRY)}; \
    *n = (int)(sizeof(table) / sizeof(table[0]));                   \
    return table;                                                   \
  }

}  // namespace lasnet
