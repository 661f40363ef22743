// The tiled schedule of the sparse bottleneck for the deep stages (14x14x1024 and 7x7x2048 in
// ResNet-101), where the weights (2.2 / 8.9 MB) dwarf what one workgroup computes on and the fused
// kernel spends its time streaming all of them through every CU.
//
// This is the paper's own operator split (Sec. 3.4 / App. B.1): conv1 is a convolution of its own
// over the map, the gather is fused into the 3x3 convolution, the scatter into the residual add;
// y1 and y2 pass through device memory (a workspace).  Three kernels, every one cut into
// (pixels of one image group) x (a slice of the output channels) per workgroup, so a workgroup
// reads only its slice of the weights while the few hundred KB of activations it needs sit in LDS:
//
//   T1  y1[p][:]  = ReLU(b1 + W1 x[p][:])    p = pixels within one pixel of an active patch (the
//                                             "needed" pixels; all of them at high activation rates)
//   T2  y2[r][:]  = ReLU(b2 + sum over the 9 taps W2[tap] y1[nbr(r, tap)][:])   r = active pixels;
//                   the group's y1 rows are loaded into LDS once and every tap reads them there
//   T3  out[p(r)] = x[p(r)] + b3 + W3 y2[r][:]                     one rounding, after the add
//
// An image group is IMGS consecutive images (1 at 14x14, 2 at 7x7): neighbourhoods never cross an
// image, so a group's rows of y1 are all a T2 workgroup needs.  Which cells are active is a byte
// mask per group: T1 builds it from the index list (every T1 workgroup scans the list for its own
// group's cells; the result does not depend on the list's order) and leaves it in the workspace for
// T2 and T3, which derive the same ascending pixel order from it.
//
// The GEMM cores are the fused kernel's phases (conv1_core / conv2_core / conv3_core), here with
// one wave per SIMD and 4 channel tiles per wave where the shape allows: D[channel][pixel] with
// v_mfma_f32_16x16x32_bf16, activations from LDS, weights as prepacked A-fragments from L2.
#pragma once
#include "bottleneck_mfma.hpp"

namespace lasnet {
namespace {

constexpr int kTiledRows = 112;                 // rows (pixels) one GEMM pass of conv1 / conv3 holds: 7 MFMA blocks
constexpr int kConv2Rows = 128;                 // ... of conv2: 8 blocks

// C, M: block shape.  IMGS: images per group.  GPXMAX: most pixels a group may have (IMGS*H*W of the
// call must not exceed it).  NSL1/2/3: slices the output channels of conv1/2/3 are cut into.
template <int C_, int M_, int IMGS_, int GPXMAX_, int NSL1_, int NSL2_, int NSL3_>
struct TiledCfg {
  static constexpr int C = C_, M = M_, IMGS = IMGS_, GPXMAX = GPXMAX_;
  static constexpr int NSL1 = NSL1_, NSL2 = NSL2_, NSL3 = NSL3_;
  static constexpr int NW = 4, NT = 256;
  static constexpr int TC1 = M / NSL1, TC2 = M / NSL2, TC3 = C / NSL3;   // channels per workgroup
  static constexpr int CMMAX = GPXMAX;                                      // cells per group <= pixels per group
  static constexpr size_t PACKED_ELEMS = (size_t)M * C * 2 + 9 * (size_t)M * M;
  static_assert(GPXMAX <= 256, "one thread per pixel of a group when the pixel lists are built");
  static_assert(GPXMAX % 2 == 0, "two 512-byte rows per load instruction");

  // ---- what the phase functions ask of a configuration -----------------------------------
  struct K1 {                                   // conv1_core
    static constexpr int C = C_, M = M_, NW = 4, NT = 256, KC = 64, NSTG = 8, WD = 3;
    static constexpr bool Y1_IN_XS = false, Y1_TO_GLOBAL = true;           // y1 rows go straight to memory
    static constexpr int YG_PITCH = M;
    static constexpr int WR1 = 1, WC1 = 4, NBW1 = TC1 / 16 / WC1;
    static constexpr int R1MAX = kTiledRows;
    static constexpr int LDX = KC, XMASK = KC / 8 - 1, STAGE_ELEMS = R1MAX * LDX;
    static constexpr int NCH = C / KC, XD = NCH <= NSTG ? NCH : NSTG - 1;
    static constexpr int LDY = TC1, YMASK = LDY / 8 - 1 < 15 ? LDY / 8 - 1 : 15;
    static constexpr int W_KSTEP_BYTES = M * 64;
    static constexpr unsigned W1_BYTES = M * C * 2;
    static_assert(TC1 % 64 == 0 && (LDY & (LDY - 1)) == 0 && C % (2 * KC) == 0, "conv1 tile");
    // LDS map
    static constexpr int OFF_ROWPIX = 0;                                   // int[R1MAX]
    static constexpr int OFF_CM = OFF_ROWPIX + R1MAX * 4;                  // uint8[CMMAX]
    static constexpr int OFF_MISC = (OFF_CM + CMMAX + 15) / 16 * 16;       // int[8]
    static constexpr int OFF_BIAS = OFF_MISC + 32;                         // float[TC1]
    static constexpr int OFF_XS = OFF_BIAS + TC1 * 4;
    static constexpr int LDS_BYTES = OFF_XS + NSTG * STAGE_ELEMS * 2 + 1024;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  };
  struct K2 {                                   // conv2_core: every output pixel is a 1x1 "patch" with a 3x3 window
    static constexpr int M = M_, S = 1, T = 3, WW = 9, NW = 4, NT = 256;
    static constexpr int WR2 = 1, WC2 = 4, NBW2 = TC2 / 16 / WC2, MS = M / 32, RD2 = 12;
    static constexpr bool ACTS_BARRIER = true, Y2_TO_GLOBAL = true;        // y2 rows go straight to memory
    static constexpr int YG_PITCH = M;
    static constexpr int ZROW = GPXMAX;                                    // the all-zero y1 row
    static constexpr int LDY = M, YMASK = 15, LDY2 = TC2, YMASK2 = 15;
    static constexpr int W_KSTEP_BYTES = M * 64;
    static constexpr unsigned W2_BYTES = 9 * M * M * 2;
    static_assert(TC2 % 64 == 0 && (9 * MS) % RD2 == 0 && M % 128 == 0, "conv2 tile");
    static constexpr int OFF_Y1 = 0;                                       // [(GPXMAX + 1)][M] bf16
    static constexpr int OFF_WINROW = OFF_Y1 + (GPXMAX + 1) * LDY * 2;     // short[GPXMAX * 9]
    static constexpr int OFF_PLIST = (OFF_WINROW + GPXMAX * 18 + 15) / 16 * 16;   // int[GPXMAX]: h << 16 | w << 8 | local pixel
    static constexpr int OFF_CM = OFF_PLIST + GPXMAX * 4;                  // uint8[CMMAX]
    static constexpr int OFF_MISC = (OFF_CM + CMMAX + 15) / 16 * 16;       // int[8]
    static constexpr int OFF_BIAS = OFF_MISC + 32;                         // float[TC2]
    static constexpr int LDS_BYTES = OFF_BIAS + TC2 * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  };
  struct K3 {                                   // conv3_core
    static constexpr int C = C_, M = M_, NW = 4, NT = 256;
    static constexpr int WR3 = 1, WC3 = 4, NBT3 = TC3 / 16 / WC3, NB3 = 4, RD3 = 4, MS = M / 32;
    static constexpr bool ACTS_BARRIER = true;
    static constexpr int LDY = M, YMASK = 15;
    static constexpr unsigned W3_BYTES = C * M * 2;
    static_assert(NBT3 % NB3 == 0 && MS % RD3 == 0, "conv3 tile");
    static constexpr int OFF_Y2 = 0;                                       // [kTiledRows][M] bf16
    static constexpr int OFF_TR = OFF_Y2 + kTiledRows * LDY * 2;           // 2 KiB per wave: store transposes
    static constexpr int OFF_PIXQ = OFF_TR + NW * 2048;                    // int[kTiledRows]: this pass
    static constexpr int OFF_PIXALL = OFF_PIXQ + kTiledRows * 4;           // int[GPXMAX]: the group's active pixels
    static constexpr int OFF_CM = OFF_PIXALL + GPXMAX * 4;                 // uint8[CMMAX]
    static constexpr int OFF_MISC = (OFF_CM + CMMAX + 15) / 16 * 16;       // int[8]
    static constexpr int OFF_BIAS = OFF_MISC + 32;                         // float[C]
    static constexpr int LDS_BYTES = OFF_BIAS + C * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
  };
  // the weight repack (pack_weights_kernel) reads these
  static constexpr int MS = M / 32, NBW1 = K1::NBW1, NBW2 = K2::NBW2, NBT3 = K3::NBT3, NB3 = K3::NB3;
};

// Run-time geometry of the grouping (by value into the kernels).  Pixel and cell coordinates inside a
// group are below 256, so divisions by hw, W and S are a multiply and a shift: a / d = (a * m) >> 16 with
// m = 65536 / d + 1, exact for a < 256 and d <= 256.
struct TiledGeom {
  int ngroups;       // ceil(N / IMGS)
  int hw;            // H * W
  int cpi;           // cells per image, G * GW
  int nt1;           // conv1 tiles per group
  int t1px;          // pixels per conv1 tile (<= kTiledRows)
  int m_hw, m_w, m_s;   // the multipliers for hw, W, S
};
inline int div_magic(int d) { return 65536 / d + 1; }
__device__ __forceinline__ int mdiv(int a, int m) { return (a * m) >> 16; }

// A pixel of a group: local image, row, column; and whether its cell is active.
struct GroupPixel { int li, h, w; };
__device__ __forceinline__ GroupPixel group_pixel(int p, const Geom& g, const TiledGeom& tg) {
  GroupPixel r;
  r.li = mdiv(p, tg.m_hw);
  const int rem = p - r.li * tg.hw;
  r.h = mdiv(rem, tg.m_w);
  r.w = rem - r.h * g.W;
  return r;
}
__device__ __forceinline__ int cell_of(const GroupPixel& q, int h, int w, const Geom& g, const TiledGeom& tg) {
  return q.li * tg.cpi + mdiv(h, tg.m_s) * g.GW + mdiv(w, tg.m_s);
}

// Workgroup b -> (unit, slice): the NSL slices of a unit are consecutive workgroups of ONE XCD
// (workgroups are dealt round-robin to the 8 XCDs, each with its own L2), so what the slices share
// -- the unit's activations -- is fetched into one L2 once.
__device__ __forceinline__ bool unit_and_slice(int nunits, int nsl, int& unit, int& slice) {
  const int xcd = (int)blockIdx.x & 7, j = (int)blockIdx.x >> 3;
  unit = (j / nsl) * 8 + xcd;
  slice = j % nsl;
  return unit < nunits;
}
inline int tiled_grid(int nunits, int nsl) { return (nunits + 7) / 8 * 8 * nsl; }

// The byte mask of one group's cells -> LDS, in two steps so that a kernel can put its long prefetches
// between them: a wave's loads complete in issue order, so whatever is requested BEFORE these small
// loads delays them, and whatever is requested after them (and before the wait) flies along.
// Source: all ones (no list = every cell active), a mask in memory (the caller's or the one T1 left:
// one byte per thread, a group has at most 256 cells), or the index list itself, scanned for this
// group's cells.  The list has room for P entries whatever the count is: its first 8192 entries are
// requested together with the count (one round trip instead of two), four per load; what the count
// excludes is dropped afterwards.
struct CellMaskReq {
  static constexpr int SPEC = 8;
  int4 v[SPEC];
  int cnt;
  unsigned char b;
  bool all_active, by_mask, aligned;
};
__device__ __forceinline__ void cell_mask_request(CellMaskReq& r, int ncell, int cell0, int P,
                                                  const int32_t* __restrict__ idx, const int32_t* __restrict__ count,
                                                  const uint8_t* __restrict__ mask, bool all_active, int tid) {
  r.all_active = all_active;
  r.by_mask = !all_active && mask != nullptr;
  r.aligned = !all_active && !mask && ((size_t)idx & 15) == 0;
  r.b = 0;
  r.cnt = 0;
  if (r.by_mask) {
    if (tid < ncell) r.b = mask[cell0 + tid];
  } else if (!all_active) {
    r.cnt = *count;
    if (r.aligned) {
      const int4* idx4 = reinterpret_cast<const int4*>(idx);
      const int cap4 = P >> 2;
#pragma unroll
      for (int u = 0; u < CellMaskReq::SPEC; ++u) {
        const int e = tid + u * 256;
        r.v[u] = e < cap4 ? idx4[e] : int4{-1, -1, -1, -1};
      }
    }
  }
}
__device__ __forceinline__ void cell_mask_finish(const CellMaskReq& r, AS_LDS unsigned char* cm, int ncell, int cell0,
                                                 int P, const int32_t* __restrict__ idx, int tid) {
  if (r.all_active) {
    for (int i = tid; i < ncell; i += 256) cm[i] = 1;
  } else if (r.by_mask) {
    if (tid < ncell) cm[tid] = r.b ? 1 : 0;
  } else {
    auto mark = [&](int c) { if ((unsigned)(c - cell0) < (unsigned)ncell) cm[c - cell0] = 1; };
    for (int i = tid; i < ncell; i += 256) cm[i] = 0;
    __syncthreads();
    const int nact = uni(min(r.cnt, P));
    int done = 0;                                          // entries the requested loads cover
    if (r.aligned) {
#pragma unroll
      for (int u = 0; u < CellMaskReq::SPEC; ++u) {
        const int e4 = (tid + u * 256) * 4;
        if (e4 + 0 < nact) mark(r.v[u].x);
        if (e4 + 1 < nact) mark(r.v[u].y);
        if (e4 + 2 < nact) mark(r.v[u].z);
        if (e4 + 3 < nact) mark(r.v[u].w);
      }
      done = min(CellMaskReq::SPEC * 1024, (P >> 2) * 4);
    }
    for (int e = done + tid; e < nact; e += 256) mark(idx[e]);
  }
  __syncthreads();
}

// Ascending compaction of a predicate over the first 256 threads' items (item = thread id):
// returns the item's position among the set ones (or -1) and the total, through 4 ints of LDS.
__device__ __forceinline__ int compact256(bool on, AS_LDS int* wtot, int tid, int& total) {
  const unsigned long long b = __ballot(on);
  const int lane = tid & 63, wv = tid >> 6;
  const int before = __popcll(b & ((1ull << lane) - 1ull));
  if (lane == 0) wtot[wv] = __popcll(b);
  __syncthreads();
  int base = 0;
  total = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int t = wtot[k];
    base += k < wv ? t : 0;
    total += t;
  }
  __syncthreads();                              // wtot may be reused
  return on ? base + before : -1;
}

// Rows of one GEMM pass when `total` rows are cut into passes of at most `cap`: near-equal passes,
// whole 16-row blocks.
__device__ __forceinline__ int pass_rows(int total, int cap) {
  const int npass = (total + cap - 1) / cap;
  return ((total + npass - 1) / npass + 15) & ~15;
}

// Rows [0, nrows) of a row-major bf16 matrix with M columns -> LDS rows 0.. (pitch M, 16-byte chunks
// XOR-swizzled with the row's low bits), by direct global->LDS loads that are left in flight.  One load
// instruction fills 1 KiB of LDS (RPI rows); the lane picks the global chunk that belongs at the
// position it writes; a ragged last piece re-reads the last row.
template <int M>
__device__ __forceinline__ void rows_to_lds_async(const AS_GLOBAL __bf16* src0, int nrows, AS_LDS __bf16* dst,
                                                  int wave, int lane) {
  constexpr int ROWB = M * 2, RPI = 1024 / ROWB, CPR = ROWB / 16;
  static_assert(RPI >= 1 && 1024 % ROWB == 0, "whole rows per load instruction");
  const int npiece = (nrows + RPI - 1) / RPI;
  const int lrow = lane / CPR, cpos = lane % CPR;
  for (int pc = wave; pc < npiece; pc += 4) {
    const int keyrow = pc * RPI + lrow;
    const int row = min(keyrow, nrows - 1);
    const AS_GLOBAL __bf16* src = src0 + (size_t)row * M + ((cpos ^ (keyrow & 15)) << 3);
    const unsigned lds_addr = uni((int)(unsigned)(size_t)(dst + (size_t)pc * 512));
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_addr) : "memory");
  }
}
// A wave must not end while its direct loads to LDS are in flight (the LDS could already be another
// workgroup's).
__device__ __forceinline__ void drain_vm() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---------------------------------------------------------------------------------------- T1
template <class TC>
__global__ __launch_bounds__(256, 1) void tiled_conv1_kernel(
    Geom g, TiledGeom tg, const __bf16* __restrict__ x, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ count, const uint8_t* __restrict__ mask_in, uint8_t* __restrict__ mask_ws,
    const __bf16* __restrict__ W1p, const float* __restrict__ b1, __bf16* __restrict__ y1g) {
  using K = typename TC::K1;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int unit, slice;
  if (!unit_and_slice(tg.ngroups * tg.nt1, TC::NSL1, unit, slice)) return;
  const int tid = threadIdx.x, wave = uni(tid >> 6);
  const int group = unit / tg.nt1, tile = unit - group * tg.nt1;
  const int img0 = group * TC::IMGS, nimg = min(TC::IMGS, g.N - img0);
  const int npx = nimg * tg.hw, ncell = nimg * tg.cpi, cell0 = img0 * tg.cpi;
  AS_LDS int* rowpix = (AS_LDS int*)(smem + K::OFF_ROWPIX);
  AS_LDS unsigned char* cm = (AS_LDS unsigned char*)(smem + K::OFF_CM);
  AS_LDS int* misc = (AS_LDS int*)(smem + K::OFF_MISC);
  AS_LDS float* b1s = (AS_LDS float*)(smem + K::OFF_BIAS);
  AS_LDS __bf16* xs = (AS_LDS __bf16*)(smem + K::OFF_XS);

  // Requested in this order: the list (or mask) and the bias, then the first weights; only then is the
  // list waited for, so the weights arrive while it is being read.
  const bool all_active = idx == nullptr;
  CellMaskReq req;
  cell_mask_request(req, ncell, cell0, g.P, idx, count, mask_in, all_active, tid);
  const float bias_v = tid < TC::TC1 ? b1[slice * TC::TC1 + tid] : 0.f;
  static_assert(TC::TC1 <= 256, "one bias per thread");
  __builtin_amdgcn_sched_barrier(0);
  const g_bf16_p W1s = (g_bf16_p)(W1p + (size_t)slice * (TC::TC1 / 16) * 512);
  Conv1Ring<K> ring;
  conv1_ring_fill<K>(ring, W1s, tid, wave);
  __builtin_amdgcn_sched_barrier(0);
  if (tid < TC::TC1) b1s[tid] = bias_v;
  cell_mask_finish(req, cm, ncell, cell0, g.P, idx, tid);
  if (mask_ws && slice == 0 && tile == 0)
    for (int i = tid; i < ncell; i += 256) mask_ws[cell0 + i] = cm[i];

  // the tile's pixels that lie within one pixel of an active cell, ascending
  const int p = tile * tg.t1px + tid;
  bool need = false;
  if (tid < tg.t1px && p < npx) {
    const GroupPixel q = group_pixel(p, g, tg);
#pragma unroll
    for (int dy = -1; dy <= 1; ++dy)
#pragma unroll
      for (int dx = -1; dx <= 1; ++dx) {
        const int hh = q.h + dy, ww = q.w + dx;
        if ((unsigned)hh < (unsigned)g.H && (unsigned)ww < (unsigned)g.W) need |= cm[cell_of(q, hh, ww, g, tg)] != 0;
      }
  }
  int U;
  const int pos = compact256(need, misc, tid, U);
  if (U == 0) return;                                      // uniform: nothing near this tile is active
  if (pos >= 0) rowpix[pos] = img0 * tg.hw + p;
  __syncthreads();
  const int nblk = (U + 15) >> 4;
  for (int r = U + tid; r < nblk * 16; r += 256) rowpix[r] = rowpix[0];   // padding rows: loaded, computed, not stored
  __syncthreads();

  dispatch_count<1, kTiledRows / 16>(nblk, [&](auto nb) {
    conv1_core<K, decltype(nb)::value, true>(ring, (g_bf16_p)x, W1s, (l_f32_cp)b1s, (l_i32_cp)rowpix, (l_bf16_p)xs,
                                             (l_bf16_p)xs, tid, wave, (AS_GLOBAL __bf16*)y1g + slice * TC::TC1, U);
  });
}

// ---------------------------------------------------------------------------------------- T2
template <class TC>
__global__ __launch_bounds__(256, 1) void tiled_conv2_kernel(
    Geom g, TiledGeom tg, const uint8_t* __restrict__ mask, int all_active,
    const __bf16* __restrict__ W2p, const float* __restrict__ b2, const __bf16* __restrict__ y1g,
    __bf16* __restrict__ y2g) {
  using K = typename TC::K2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int group, slice;
  if (!unit_and_slice(tg.ngroups, TC::NSL2, group, slice)) return;
  const int tid = threadIdx.x, wave = uni(tid >> 6), lane = tid & 63;
  const int img0 = group * TC::IMGS, nimg = min(TC::IMGS, g.N - img0);
  const int npx = nimg * tg.hw, ncell = nimg * tg.cpi, cell0 = img0 * tg.cpi;
  AS_LDS __bf16* y1s = (AS_LDS __bf16*)(smem + K::OFF_Y1);
  AS_LDS short* winrow = (AS_LDS short*)(smem + K::OFF_WINROW);
  AS_LDS int* plist = (AS_LDS int*)(smem + K::OFF_PLIST);
  AS_LDS unsigned char* cm = (AS_LDS unsigned char*)(smem + K::OFF_CM);
  AS_LDS int* misc = (AS_LDS int*)(smem + K::OFF_MISC);
  AS_LDS float* b2s = (AS_LDS float*)(smem + K::OFF_BIAS);

  // Requested in this order: the mask and the bias, the first weights, and -- once the mask has arrived
  // -- the group's y1 rows -> LDS (row = local pixel; rows that no active pixel needs were never written
  // by T1: loaded all the same, never read), which are awaited inside conv2_core.
  CellMaskReq req;
  cell_mask_request(req, ncell, cell0, g.P, nullptr, nullptr, mask, all_active != 0, tid);
  const float bias_v = tid < TC::TC2 ? b2[slice * TC::TC2 + tid] : 0.f;
  static_assert(TC::TC2 <= 256, "one bias per thread");
  __builtin_amdgcn_sched_barrier(0);
  const g_bf16_p W2s = (g_bf16_p)(W2p + (size_t)slice * (TC::TC2 / 16) * 512);
  Conv2Ring<K> ring;
  conv2_ring_fill<K>(ring, W2s, tid, wave);
  __builtin_amdgcn_sched_barrier(0);
  if (tid < TC::TC2) b2s[tid] = bias_v;
  cell_mask_finish(req, cm, ncell, cell0, g.P, nullptr, tid);
  rows_to_lds_async<TC::M>((const AS_GLOBAL __bf16*)y1g + (size_t)img0 * tg.hw * TC::M, npx, y1s, wave, lane);
  for (int i = tid; i < K::LDY / 8; i += 256)
    *reinterpret_cast<AS_LDS bf16x8*>(y1s + K::ZROW * K::LDY + i * 8) = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
  // the group's active pixels, ascending: output row q <-> local pixel plist[q] (with its coordinates)
  bool on = false;
  GroupPixel me{0, 0, 0};
  if (tid < npx) {
    me = group_pixel(tid, g, tg);
    on = cm[cell_of(me, me.h, me.w, g, tg)] != 0;
  }
  int A;
  const int q = compact256(on, misc, tid, A);
  if (A == 0) { drain_vm(); return; }                      // uniform
  if (q >= 0) plist[q] = me.h << 16 | me.w << 8 | tid;
  __syncthreads();                                         // plist is complete
  // row of each of the 9 window positions of every output pixel (the zero row outside the image)
  for (int t = tid; t < A * 9; t += 256) {
    const int qq = t / 9, tap = t - qq * 9;
    const int e = plist[qq], ph = e >> 16, pw = (e >> 8) & 255, pl = e & 255;
    const int dy = tap / 3 - 1, dx = tap - (tap / 3) * 3 - 1;
    winrow[t] = ((unsigned)(ph + dy) < (unsigned)g.H && (unsigned)(pw + dx) < (unsigned)g.W)
                    ? (short)(pl + dy * g.W + dx) : (short)K::ZROW;
  }
  // (no barrier here: conv2_core has one on entry)

  const int prows = pass_rows(A, kConv2Rows);
  AS_GLOBAL __bf16* y2dst = (AS_GLOBAL __bf16*)y2g + (size_t)group * TC::IMGS * tg.hw * TC::M + slice * TC::TC2;
  for (int p0 = 0; p0 < A; p0 += prows) {
    const int nq = min(prows, A - p0);
    dispatch_count<1, kConv2Rows / 16>((nq + 15) >> 4, [&](auto nb) {
      conv2_core<K, decltype(nb)::value, true>(ring, W2s, (l_f32_cp)b2s, (l_i16_cp)(winrow + p0 * 9), (l_bf16_cp)y1s,
                                               (l_bf16_p)nullptr, nq, tid, wave, y2dst + (size_t)p0 * TC::M);
    });
  }
  drain_vm();                                              // (the ring's wrapped refills)
}

// ---------------------------------------------------------------------------------------- T3
template <class TC>
__global__ __launch_bounds__(256, 1) void tiled_conv3_kernel(
    Geom g, TiledGeom tg, const uint8_t* __restrict__ mask, int all_active, const __bf16* x,
    const __bf16* __restrict__ W3p, const float* __restrict__ b3, const __bf16* __restrict__ y2g,
    __bf16* out, int post_relu) {                          // out may be x: a lane reads and writes the same elements
  using K = typename TC::K3;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int group, slice;
  if (!unit_and_slice(tg.ngroups, TC::NSL3, group, slice)) return;
  const int tid = threadIdx.x, wave = uni(tid >> 6), lane = tid & 63;
  const int img0 = group * TC::IMGS, nimg = min(TC::IMGS, g.N - img0);
  const int npx = nimg * tg.hw, ncell = nimg * tg.cpi, cell0 = img0 * tg.cpi;
  AS_LDS __bf16* y2s = (AS_LDS __bf16*)(smem + K::OFF_Y2);
  AS_LDS __bf16* trs = (AS_LDS __bf16*)(smem + K::OFF_TR);
  AS_LDS int* pixq = (AS_LDS int*)(smem + K::OFF_PIXQ);
  AS_LDS int* pixall = (AS_LDS int*)(smem + K::OFF_PIXALL);
  AS_LDS unsigned char* cm = (AS_LDS unsigned char*)(smem + K::OFF_CM);
  AS_LDS int* misc = (AS_LDS int*)(smem + K::OFF_MISC);
  AS_LDS float* b3s = (AS_LDS float*)(smem + K::OFF_BIAS);

  // Requested in this order: the mask and the bias, the first weights, and -- once the mask has arrived
  // -- the first pass's y2 rows (before the active count is known: rows past it are never used; the
  // group's y2 area has room for every pixel), which are awaited inside conv3_core.
  CellMaskReq req;
  cell_mask_request(req, ncell, cell0, g.P, nullptr, nullptr, mask, all_active != 0, tid);
  constexpr int NBV = TC::C / 256;
  float bias_v[NBV];
#pragma unroll
  for (int u = 0; u < NBV; ++u) bias_v[u] = b3[tid + u * 256];
  __builtin_amdgcn_sched_barrier(0);
  Conv3Ring<K> ring;
  conv3_ring_fill<K>(ring, (g_bf16_p)W3p, tid, wave, slice * K::WC3);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < NBV; ++u) b3s[tid + u * 256] = bias_v[u];
  cell_mask_finish(req, cm, ncell, cell0, g.P, nullptr, tid);
  const AS_GLOBAL __bf16* y2src = (const AS_GLOBAL __bf16*)y2g + (size_t)group * TC::IMGS * tg.hw * TC::M;
  rows_to_lds_async<TC::M>(y2src, min(kTiledRows, npx), y2s, wave, lane);
  bool on = false;
  if (tid < npx) {
    const GroupPixel me = group_pixel(tid, g, tg);
    on = cm[cell_of(me, me.h, me.w, g, tg)] != 0;
  }
  int A;
  const int q = compact256(on, misc, tid, A);
  if (A == 0) { drain_vm(); return; }                      // uniform
  if (q >= 0) pixall[q] = img0 * tg.hw + tid;              // same order as T2's rows
  __syncthreads();

  const int prows = pass_rows(A, kTiledRows);
  for (int p0 = 0; p0 < A; p0 += prows) {
    const int nq = min(prows, A - p0);
    const int nblk = (nq + 15) >> 4;
    if (p0 > 0) rows_to_lds_async<TC::M>(y2src + (size_t)p0 * TC::M, nq, y2s, wave, lane);
    for (int i = tid; i < nblk * 16; i += 256) pixq[i] = i < nq ? pixall[p0 + i] : -1;
    dispatch_count<1, kTiledRows / 16>(nblk, [&](auto nb) {
      conv3_core<K, decltype(nb)::value, true>(ring, (g_bf16_p)x, (g_bf16_p)W3p, (l_f32_cp)b3s, (l_i32_cp)pixq,
                                               (l_bf16_cp)y2s, (l_bf16_p)trs, (AS_GLOBAL __bf16*)out, post_relu, tid,
                                               wave, slice * K::WC3);
    });
    if (p0 + prows < A) __syncthreads();                   // y2s and pixq are rewritten by the next pass
  }
  drain_vm();                                              // (the ring's wrapped refills)
}

// ---------------------------------------------------------------------------------------- host
// Workspace of one call: the group cell masks, y1 for every pixel, y2 for every pixel (capacity).
template <class TC>
size_t tiled_workspace_bytes(const Geom& g) {
  const size_t px = (size_t)g.N * g.H * g.W;
  const size_t groups = ((size_t)g.N + TC::IMGS - 1) / TC::IMGS;
  return (((size_t)g.P + 255) / 256) * 256 + px * TC::M * 2 + groups * TC::IMGS * g.H * g.W * TC::M * 2;
}

template <class TC>
bool tiled_takes(const Geom& g) {
  return g.C == TC::C && g.M == TC::M && TC::IMGS * g.H * g.W <= TC::GPXMAX;
}

template <class TC>
hipError_t prepare_tiled() {
  static std::atomic<unsigned long long> done[3];
  if (hipError_t e = allow_dynamic_lds((const void*)tiled_conv1_kernel<TC>, TC::K1::LDS_BYTES, done[0]); e != hipSuccess)
    return e;
  if (hipError_t e = allow_dynamic_lds((const void*)tiled_conv2_kernel<TC>, TC::K2::LDS_BYTES, done[1]); e != hipSuccess)
    return e;
  return allow_dynamic_lds((const void*)tiled_conv3_kernel<TC>, TC::K3::LDS_BYTES, done[2]);
}

template <class TC>
hipError_t pack_tiled(const void* W1, const void* W2, const void* W3, void* packed, hipStream_t st) {
  hipLaunchKernelGGL(pack_weights_kernel<TC>, dim3((unsigned)((TC::PACKED_ELEMS / 8 + 255) / 256)), dim3(256), 0,
                     st, (const __bf16*)W1, (const __bf16*)W2, (const __bf16*)W3, (__bf16*)packed);
  return hipGetLastError();
}

// cellmask: the masker's byte mask of the same call, if the caller has it (saves T1 the scan of the
// list), else nullptr.  idx == nullptr: every cell active.
template <class TC>
hipError_t launch_tiled(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                        const uint8_t* cellmask, const void* packed, const float* b1, const float* b2,
                        const float* b3, void* out, bool post_relu, void* workspace, hipStream_t st) {
  if (!tiled_takes<TC>(g) || !workspace) return hipErrorInvalidValue;
  if (hipError_t e = prepare_tiled<TC>(); e != hipSuccess) return e;
  TiledGeom tg;
  tg.ngroups = (g.N + TC::IMGS - 1) / TC::IMGS;
  tg.hw = g.H * g.W;
  tg.cpi = g.G * g.GW;
  const int gpx = TC::IMGS * tg.hw;
  tg.nt1 = (gpx + kTiledRows - 1) / kTiledRows;
  tg.t1px = (gpx + tg.nt1 - 1) / tg.nt1;
  tg.m_hw = div_magic(tg.hw);
  tg.m_w = div_magic(g.W);
  tg.m_s = div_magic(g.S);
  unsigned char* ws = (unsigned char*)workspace;
  uint8_t* mask_ws = ws;
  __bf16* y1g = (__bf16*)(ws + (((size_t)g.P + 255) / 256) * 256);
  __bf16* y2g = y1g + (size_t)g.N * tg.hw * TC::M;
  const __bf16* p1 = (const __bf16*)packed;
  const __bf16* p2 = p1 + (size_t)TC::M * TC::C;
  const __bf16* p3 = p2 + 9 * (size_t)TC::M * TC::M;
  const bool all = idx == nullptr;
  const uint8_t* mask_src = all ? nullptr : (cellmask ? cellmask : mask_ws);
  hipLaunchKernelGGL(tiled_conv1_kernel<TC>, dim3(tiled_grid(tg.ngroups * tg.nt1, TC::NSL1)), dim3(256),
                     TC::K1::LDS_BYTES, st, g, tg, (const __bf16*)x, idx, count, all ? nullptr : cellmask,
                     (all || cellmask) ? nullptr : mask_ws, p1, b1, y1g);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  hipLaunchKernelGGL(tiled_conv2_kernel<TC>, dim3(tiled_grid(tg.ngroups, TC::NSL2)), dim3(256), TC::K2::LDS_BYTES, st,
                     g, tg, mask_src, (int)all, p2, b2, (const __bf16*)y1g, y2g);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  hipLaunchKernelGGL(tiled_conv3_kernel<TC>, dim3(tiled_grid(tg.ngroups, TC::NSL3)), dim3(256), TC::K3::LDS_BYTES, st,
                     g, tg, mask_src, (int)all, (const __bf16*)x, p3, b3, (const __bf16*)y2g, (__bf16*)out,
                     (int)post_relu);
  return hipGetLastError();
}

}  // namespace
}  // namespace lasnet
