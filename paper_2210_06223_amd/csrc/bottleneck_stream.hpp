// Streaming, weight-stationary variant of the fused sparse bottleneck for the first ResNet
// stage (C = 256, M = 64, S = 8), where the block is memory-bound: 137 KB of weights against
// 103 MB maps.
//
// A persistent workgroup (4 waves, one per SIMD of its CU, so each may use the whole register
// file) keeps ALL of W1, W2, W3 in registers as MFMA A-fragments and walks through its run of the
// active-patch list one patch at a time (Sec. 3.4 / App. B.1: gather fused into the first
// convolution, scatter into the residual add).  The waves form a 2 x 2 grid: a wave row takes every
// other 16-pixel block, a wave column half of the output channels, so a B fragment read from LDS
// feeds two (conv1, conv2) or eight (conv3) MFMAs; 272 registers per lane hold the wave's weights.
// Per patch:
//
//   top      the (S+2)x(S+2) window of the NEXT patch is requested global -> LDS (the other half
//            of a double buffer), so HBM works while this patch is computed; nothing else in the
//            loop loads from global memory (weights in registers, biases and patch origins in LDS,
//            the residual is the window's own interior), so the only wait for memory is one
//            per patch, a whole patch after the request
//   conv1    y1 = ReLU(W1 x + b1) on the 100 window positions; positions outside the image
//            get y1 = 0 (the 3x3 pads conv1's output)                     -> LDS, row = wy*16 + wx
//   conv2    3x3 from LDS, rows addressed arithmetically (no lookup table) -> y2 in LDS
//   conv3    + b3 + residual from the x window in LDS, one rounding, whole-line streaming stores
//
// The pixel of every window position of a patch (or -1 outside the image) is tabulated in LDS two
// patches ahead, off the critical path, from the patch origins decoded once at the start.
//
// It reads the packed weight buffer of the Cfg with WC = 4 wave columns and NB3 = 4 (the layout
// pack_weights_kernel writes for the stage-1 instantiations), so it is a drop-in launcher: a wave
// column here takes two of that layout's columns.
#pragma once
#include "bottleneck_mfma.hpp"

namespace lasnet {
namespace {

template <int C_, int M_, int S_>
struct StreamCfg {
  static constexpr int C = C_, M = M_, S = S_;
  static constexpr int NW = 4, NT = NW * 64, WR = 2, WC = 2;   // one wave per SIMD: 512 registers each
  static constexpr int T = S + 2, WW = T * T;              // window side, window positions
  static constexpr int R1 = roundup(WW, 16), R1B = R1 / 16; // x rows in LDS / conv1 row blocks
  static constexpr int RB1 = cdiv(R1B, WR);                 // conv1 row blocks per wave row
  static constexpr int Q = S * S, QB = Q / 16, RB2 = QB / WR;   // output pixels, their blocks
  static constexpr int TP = 16;                             // y1 row = wy * TP + wx
  static constexpr int Y1ROWS = T * TP;
  static constexpr int KS1 = C / 32, KS2 = M / 32;
  static constexpr int MT = M / 16 / WC;                    // mid-channel tiles per wave (conv1, conv2)
  static constexpr int G3 = C / 64 / WC, NT3 = 4;           // conv3: groups of 4 tiles (64 channels) per wave
  static constexpr int XROW = C * 2, YROW = M * 2;          // bytes per LDS row
  static constexpr int MAXQ = 64;                           // list entries one workgroup takes
  static constexpr int XGRP = R1 / 2;                       // 1 KiB pieces (two x rows) of a window
  static constexpr int NXL = XGRP / NW;                     // x loads per wave per patch
  static constexpr int OFF_XS = 0, XS_BYTES = 2 * R1 * XROW;
  static constexpr int OFF_Y1 = OFF_XS + XS_BYTES, Y1_BYTES = Y1ROWS * YROW;
  static constexpr int OFF_Y2 = OFF_Y1 + Y1_BYTES, Y2_BYTES = Q * YROW;
  static constexpr int OFF_BIAS = OFF_Y2 + Y2_BYTES, BIAS_BYTES = (2 * M + C) * 4;
  static constexpr int OFF_PIX = OFF_BIAS + BIAS_BYTES, PIX_BYTES = 3 * 2 * R1 * 4;
  static constexpr int OFF_HDR = OFF_PIX + PIX_BYTES;       // per list entry: base pixel, h0, w0, -
  static constexpr int LDS_BYTES = OFF_HDR + MAXQ * 16;
  static_assert(M == 64 && KS2 == 2, "y rows are 128 bytes: 8 swizzle chunks");
  static_assert(XROW == 512, "an x row is 512 bytes: 32 chunks, pixel -> byte offset is a shift by 9");
  static_assert(C % (64 * WC) == 0 && M % (16 * WC) == 0, "channels split over the wave columns");
  static_assert(S == 8 && T <= TP, "64 output pixels; a window row fits the y1 pitch");
  static_assert(QB % WR == 0 && R1 % 2 == 0, "row blocks split over the wave rows");
  static_assert(XGRP % NW == 0, "every wave requests the same number of window pieces");
  static_assert(NW * 2 * 2048 <= Y1_BYTES, "conv3's transpose areas (two per wave) sit in the y1 rows");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

// Swizzle keys of the 128-byte y rows (8 chunks of 16 bytes; even and odd rows sit in different
// bank halves).  y1: a conv2 fragment read touches rows r..r+7 and r+16..r+23 -> 8 distinct
// keys among the rows of one parity.  y2: 16 consecutive rows.
__device__ __forceinline__ int y1_key(int row) { return ((row >> 1) & 3) | ((row >> 2) & 4); }
__device__ __forceinline__ int y2_key(int row) { return (row >> 1) & 7; }

template <class K, bool POST_RELU>
__global__ __launch_bounds__(K::NT, 1) void stream_bneck_kernel(
    Geom g, const __bf16* __restrict__ x, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ count, const __bf16* __restrict__ W1p, const float* __restrict__ b1,
    const __bf16* __restrict__ W2p, const float* __restrict__ b2, const __bf16* __restrict__ W3p,
    const float* __restrict__ b3, __bf16* __restrict__ out) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int C = K::C, M = K::M, S = K::S, T = K::T, WW = K::WW;
  AS_LDS char* lds = (AS_LDS char*)smem;
  AS_LDS char* xs = lds + K::OFF_XS;
  AS_LDS char* y1s = lds + K::OFF_Y1;
  AS_LDS char* y2s = lds + K::OFF_Y2;
  AS_LDS float* b1s = (AS_LDS float*)(lds + K::OFF_BIAS);
  AS_LDS float* b2s = b1s + M;
  AS_LDS float* b3s = b2s + M;
  // [3][2][R1]: pixel of each window position, -1 outside the image; then the pixel to LOAD for the
  // position (outside the image: the patch's first own pixel, so that every load is in bounds)
  AS_LDS int* pixs = (AS_LDS int*)(lds + K::OFF_PIX);
  AS_LDS int* hdr = (AS_LDS int*)(lds + K::OFF_HDR);       // window origin of each list entry

  const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lg = lane >> 4;
  const int wave = uni(tid >> 6), wr = wave / K::WC, wc = wave % K::WC;

  // ---- this workgroup's run of the list (XCD k takes a contiguous eighth of the runs) ------
  const int nact = uni(idx ? min(*count, g.P) : g.P);
  if (nact <= 0) return;
  const int nt = min((int)gridDim.x, nact);
  if ((int)blockIdx.x >= nt) return;
  const int xcd = (int)blockIdx.x & 7, jx = (int)blockIdx.x >> 3;
  const int run = xcd * (nt >> 3) + min(xcd, nt & 7) + jx;
  const int tb = (int)(((long long)run * nact) / nt);
  const int npat = (int)(((long long)(run + 1) * nact) / nt) - tb;   // <= MAXQ by the grid size

  for (int i = tid; i < npat; i += K::NT) {
    const int cell = idx ? idx[tb + i] : tb + i;
    const int n = cell / (g.G * g.GW), rem = cell - n * (g.G * g.GW);
    const int gy = rem / g.GW, gx = rem - gy * g.GW;
    int h0 = gy * S - 1, w0 = gx * S - 1, base = (n * g.H + h0) * g.W + w0;
    if ((unsigned)cell >= (unsigned)g.P) {                   // not a cell of this map: a window that lies
      h0 = w0 = -(1 << 20);                                  // wholly outside the image (nothing is stored
      base = -(g.W + 1);                                     // for it; its loads read pixel 0)
    }
    hdr[i * 4 + 0] = base;
    hdr[i * 4 + 1] = h0;
    hdr[i * 4 + 2] = w0;
  }
  for (int i = tid; i < M; i += K::NT) { b1s[i] = b1[i]; b2s[i] = b2[i]; }
  for (int i = tid; i < C; i += K::NT) b3s[i] = b3[i];

  // ---- all weights of this wave -> registers (A fragments), once ---------------------------
  bf16x8 w1[K::KS1][K::MT], w2[9 * K::KS2][K::MT], w3[K::KS2][K::G3][K::NT3];
  {
    const AS_GLOBAL bf16x8* p1 = (const AS_GLOBAL bf16x8*)W1p + lane;
    const AS_GLOBAL bf16x8* p2 = (const AS_GLOBAL bf16x8*)W2p + lane;
    const AS_GLOBAL bf16x8* p3 = (const AS_GLOBAL bf16x8*)W3p + lane;
#pragma unroll
    for (int ks = 0; ks < K::KS1; ++ks)
#pragma unroll
      for (int tt = 0; tt < K::MT; ++tt) w1[ks][tt] = p1[(ks * (M / 16) + wc * K::MT + tt) * 64];
#pragma unroll
    for (int t = 0; t < 9 * K::KS2; ++t)
#pragma unroll
      for (int tt = 0; tt < K::MT; ++tt) w2[t][tt] = p2[(t * (M / 16) + wc * K::MT + tt) * 64];
#pragma unroll
    for (int ks = 0; ks < K::KS2; ++ks)
#pragma unroll
      for (int gg = 0; gg < K::G3; ++gg)
#pragma unroll
        for (int j = 0; j < K::NT3; ++j)
          w3[ks][gg][j] = p3[(((wc * K::G3 + gg) * K::KS2 + ks) * K::NT3 + j) * 64];
  }
  // W2 and W3 live in the accumulation registers (an MFMA reads its A operand from either half of
  // the register file; other instructions only from the first 256, which stay free for W1, the
  // accumulators and the epilogues).  Without this the compiler parks them there anyway, as spills,
  // and copies each fragment back before the MFMA that uses it.
#pragma unroll
  for (int t = 0; t < 9 * K::KS2; ++t)
#pragma unroll
    for (int tt = 0; tt < K::MT; ++tt) asm volatile("" : "+a"(w2[t][tt]));
#pragma unroll
  for (int ks = 0; ks < K::KS2; ++ks)
#pragma unroll
    for (int gg = 0; gg < K::G3; ++gg)
#pragma unroll
      for (int j = 0; j < K::NT3; ++j) asm volatile("" : "+a"(w3[ks][gg][j]));
  __syncthreads();                                         // patch origins and biases are in LDS

  // pixel of every window position of list entry p (or -1): window position (wy, wx) of a window
  // that starts at (h0, w0) = (gy*S - 1, gx*S - 1) is pixel base + wy*W + wx, base = (n*H + h0)*W + w0
  auto decode = [&](int p) {
    if (tid < K::R1) {
      const int base = hdr[p * 4], h0 = hdr[p * 4 + 1], w0 = hdr[p * 4 + 2];
      const int wy = tid / T, wx = tid - wy * T;
      const bool in = tid < WW && (unsigned)(h0 + wy) < (unsigned)g.H && (unsigned)(w0 + wx) < (unsigned)g.W;
      const int px = base + wy * g.W + wx;
      pixs[(p % 3) * (2 * K::R1) + tid] = in ? px : -1;
      pixs[(p % 3) * (2 * K::R1) + K::R1 + tid] = in ? px : base + g.W + 1;
    }
  };
  // request the x window of entry p: a wave instruction fills two 512-byte rows (chunks swizzled
  // with the row's low 4 bits).  Byte offsets from x fit 32 bits (the launcher checks).
  auto issue_x = [&](int p) {
    AS_LDS const int* pl = pixs + (p % 3) * (2 * K::R1) + K::R1 + wave * 2 + (lane >> 5);
    int px[K::NXL];
#pragma unroll
    for (int u = 0; u < K::NXL; ++u) px[u] = pl[u * K::NW * 2];
    const unsigned lds0 = uni((int)(unsigned)(size_t)(xs + (p & 1) * (K::R1 * K::XROW) + wave * 1024));
#pragma unroll
    for (int u = 0; u < K::NXL; ++u) {
      {
        // row = (wave + 4u)*2 + (lane >> 5): its low 4 bits are those of wave*2 + (lane >> 5) + 8u
        const int key = (wave * 2 + (lane >> 5) + 8 * (u & 1)) & 15;
        const unsigned off = ((unsigned)px[u] << 9) + ((((lane & 31) ^ key)) << 4);
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(x),
                     "s"(lds0 + u * K::NW * 1024)
                     : "memory");
      }
    }
  };

  decode(0);
  if (npat > 1) decode(1);
  __syncthreads();
  issue_x(0);

  for (int p = 0; p < npat; ++p) {
    AS_LDS const char* xc = xs + (p & 1) * (K::R1 * K::XROW);
    AS_LDS const int* pix = pixs + (p % 3) * (2 * K::R1);
    // The window of entry p has landed (requested a whole patch ago), the previous patch's stores
    // are done and every wave has left the previous patch.  (Letting those stores stay in flight
    // here measured the same.)
    barrier_keep_vm<0>();
    if (p + 1 < npat) issue_x(p + 1);

    // ------------------------------------------------------------------ conv1
    {
      floatx4 acc[K::RB1][K::MT];
      FragRow fr[K::RB1];
#pragma unroll
      for (int i = 0; i < K::RB1; ++i) {
        // the accumulators start at the bias: the first MFMA takes it as its C operand
#pragma unroll
        for (int tt = 0; tt < K::MT; ++tt)
          acc[i][tt] = *reinterpret_cast<AS_LDS const floatx4*>(b1s + (wc * K::MT + tt) * 16 + lg * 4);
        // a wave row's last block may not exist (R1B not a multiple of WR): it recomputes the
        // last real one, and its result is dropped
        const int row = min(wr + K::WR * i, K::R1B - 1) * 16 + l16;
        fr[i] = frag_row(row, C, lg, row, 15);
      }
      // B fragments are read PF k-steps ahead of the MFMAs that use them: with one wave per SIMD
      // nothing else hides the LDS latency (deeper than 1 measured the same)
      constexpr int PF = 1;
      bf16x8 bq[PF + 1][K::RB1];
#pragma unroll
      for (int s0 = 0; s0 < PF; ++s0)
#pragma unroll
        for (int i = 0; i < K::RB1; ++i) bq[s0][i] = frag_read((const AS_LDS __bf16*)xc, fr[i], s0);
#pragma unroll
      for (int ks = 0; ks < K::KS1; ++ks) {
        if (ks + PF < K::KS1) {
#pragma unroll
          for (int i = 0; i < K::RB1; ++i)
            bq[(ks + PF) % (PF + 1)][i] = frag_read((const AS_LDS __bf16*)xc, fr[i], ks + PF);
        }
#pragma unroll
        for (int i = 0; i < K::RB1; ++i)
#pragma unroll
          for (int tt = 0; tt < K::MT; ++tt) acc[i][tt] = mfma16(w1[ks][tt], bq[ks % (PF + 1)][i], acc[i][tt]);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < K::RB1; ++i) {
        const int wp = (wr + K::WR * i) * 16 + l16;        // window position = x row
        if (wr + K::WR * i < K::R1B && wp < WW) {          // (the first test is wave-uniform)
          const bool in = pix[wp] >= 0;
          const int row = (wp / T) * K::TP + wp % T;
#pragma unroll
          for (int tt = 0; tt < K::MT; ++tt) {
            const int ch = (wc * K::MT + tt) * 16 + lg * 4;   // this lane's 4 channels of the tile
            bf16x4 o;
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = (__bf16)(in ? fmaxf(acc[i][tt][v], 0.f) : 0.f);
            *reinterpret_cast<AS_LDS bf16x4*>(y1s + row * K::YROW + (((ch >> 3) ^ y1_key(row)) << 4) + (ch & 7) * 2) = o;
          }
        }
      }
    }
    barrier_keep_vm<63>();                                 // LDS only: the next window stays in flight
    if (p + 2 < npat) decode(p + 2);                       // read after the next patch's first barrier

    // ------------------------------------------------------------------ conv2
    {
      floatx4 acc[K::RB2][K::MT];
      int r00[K::RB2];                                     // y1 row of tap (0,0)
#pragma unroll
      for (int i = 0; i < K::RB2; ++i) {
#pragma unroll
        for (int tt = 0; tt < K::MT; ++tt)
          acc[i][tt] = *reinterpret_cast<AS_LDS const floatx4*>(b2s + (wc * K::MT + tt) * 16 + lg * 4);
        const int q = (wr + K::WR * i) * 16 + l16;
        r00[i] = (q / S) * K::TP + q % S;
      }
      // both k-steps of a tap are read one tap ahead of the MFMAs that use them
      auto read_tap = [&](bf16x8 (&b)[K::RB2][K::KS2], int tap) {
#pragma unroll
        for (int i = 0; i < K::RB2; ++i) {
          const int row = r00[i] + (tap / 3) * K::TP + tap % 3;
          AS_LDS const char* rp = y1s + row * K::YROW;
          const int key = y1_key(row);
#pragma unroll
          for (int ks = 0; ks < K::KS2; ++ks)
            b[i][ks] = *reinterpret_cast<AS_LDS const bf16x8*>(rp + (((ks * 4 + lg) ^ key) << 4));
        }
      };
      bf16x8 bcur[K::RB2][K::KS2], bnxt[K::RB2][K::KS2];
      read_tap(bcur, 0);
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        if (tap + 1 < 9) read_tap(bnxt, tap + 1);
#pragma unroll
        for (int ks = 0; ks < K::KS2; ++ks)
#pragma unroll
          for (int i = 0; i < K::RB2; ++i)
#pragma unroll
            for (int tt = 0; tt < K::MT; ++tt)
              acc[i][tt] = mfma16(w2[tap * K::KS2 + ks][tt], bcur[i][ks], acc[i][tt]);
        __builtin_amdgcn_sched_barrier(0);
        if (tap + 1 < 9) {
#pragma unroll
          for (int i = 0; i < K::RB2; ++i)
#pragma unroll
            for (int ks = 0; ks < K::KS2; ++ks) bcur[i][ks] = bnxt[i][ks];
        }
      }
#pragma unroll
      for (int i = 0; i < K::RB2; ++i) {
        const int q = (wr + K::WR * i) * 16 + l16;
#pragma unroll
        for (int tt = 0; tt < K::MT; ++tt) {
          const int ch = (wc * K::MT + tt) * 16 + lg * 4;
          bf16x4 o;
#pragma unroll
          for (int v = 0; v < 4; ++v) o[v] = (__bf16)fmaxf(acc[i][tt][v], 0.f);
          *reinterpret_cast<AS_LDS bf16x4*>(y2s + q * K::YROW + (((ch >> 3) ^ y2_key(q)) << 4) + (ch & 7) * 2) = o;
        }
      }
    }
    barrier_keep_vm<63>();

    // ------------------------------------------------------------------ conv3 + residual + store
    {
      // the residual (the window's own interior) is read ahead of the MFMAs
      bf16x8 res[K::RB2][K::G3][2];
#pragma unroll
      for (int i = 0; i < K::RB2; ++i) {
        const int q = (wr + K::WR * i) * 16 + l16;
        const int wp = (q / S + 1) * T + q % S + 1;        // the pixel's own window position
#pragma unroll
        for (int gg = 0; gg < K::G3; ++gg)
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const int c8 = (wc * K::G3 + gg) * 64 + t * 32 + lg * 8;   // 8 consecutive channels (tiles 2t, 2t+1)
            res[i][gg][t] = *reinterpret_cast<AS_LDS const bf16x8*>(xc + wp * K::XROW + (((c8 >> 3) ^ (wp & 15)) << 4));
          }
      }
      floatx4 acc[K::RB2][K::G3][K::NT3];
#pragma unroll
      for (int i = 0; i < K::RB2; ++i)
#pragma unroll
        for (int gg = 0; gg < K::G3; ++gg)
#pragma unroll
          for (int j = 0; j < K::NT3; ++j)   // tile j of a group: channels (j >> 1) * 32 + lg * 8 + (j & 1) * 4 ..
            acc[i][gg][j] = *reinterpret_cast<AS_LDS const floatx4*>(
                b3s + (wc * K::G3 + gg) * 64 + (j >> 1) * 32 + lg * 8 + (j & 1) * 4);
#pragma unroll
      for (int ks = 0; ks < K::KS2; ++ks) {
#pragma unroll
        for (int i = 0; i < K::RB2; ++i) {
          const int q = (wr + K::WR * i) * 16 + l16;
          const bf16x8 b = *reinterpret_cast<AS_LDS const bf16x8*>(y2s + q * K::YROW + (((ks * 4 + lg) ^ y2_key(q)) << 4));
#pragma unroll
          for (int gg = 0; gg < K::G3; ++gg)
#pragma unroll
            for (int j = 0; j < K::NT3; ++j) acc[i][gg][j] = mfma16(w3[ks][gg][j], b, acc[i][gg][j]);
        }
      }
      // One unit = 16 pixels x 64 channels (128 bytes per pixel).  It goes through 2 KiB of the
      // wave's own LDS (y1 is dead now) so that a store instruction writes 8 whole 128-byte lines,
      // 8 consecutive lanes per line.  A wave has two such areas: the units of a row block are
      // written, then read back and stored, together.
      AS_LDS char* tr = y1s + wave * 4096;
      const int c8l = lane & 7;
#pragma unroll
      for (int i = 0; i < K::RB2; ++i) {
#pragma unroll
        for (int gg = 0; gg < K::G3; ++gg) {
          const int chb = (wc * K::G3 + gg) * 64;          // first of the unit's 64 output channels
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            bf16x8 o;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              float r0 = (float)res[i][gg][t][v] + acc[i][gg][2 * t][v];
              float r1 = (float)res[i][gg][t][4 + v] + acc[i][gg][2 * t + 1][v];
              if (POST_RELU) { r0 = fmaxf(r0, 0.f); r1 = fmaxf(r1, 0.f); }
              o[v] = (__bf16)r0;
              o[4 + v] = (__bf16)r1;
            }
            *reinterpret_cast<AS_LDS bf16x8*>(tr + gg * 2048 + l16 * 128 + (((4 * t + lg) ^ (l16 & 7)) << 4)) = o;
          }
        }
#pragma unroll
        for (int gg = 0; gg < K::G3; ++gg) {
          const int chb = (wc * K::G3 + gg) * 64;
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const int pr = half * 8 + (lane >> 3);
            const bf16x8 v = *reinterpret_cast<AS_LDS const bf16x8*>(tr + gg * 2048 + pr * 128 + ((c8l ^ (pr & 7)) << 4));
            const int qq = (wr + K::WR * i) * 16 + pr;
            const int px = pix[(qq / S + 1) * T + qq % S + 1];   // own pixels are inside the image, unless the entry was invalid
            if (px >= 0)
              __builtin_nontemporal_store(v, reinterpret_cast<AS_GLOBAL bf16x8*>((AS_GLOBAL __bf16*)out + (size_t)px * C + chb + c8l * 8));
          }
        }
      }
    }
  }
}

template <class K>
hipError_t prepare_stream() {
  static std::atomic<unsigned long long> lds_allowed[2];
  if (hipError_t e = allow_dynamic_lds((const void*)stream_bneck_kernel<K, false>, K::LDS_BYTES, lds_allowed[0]);
      e != hipSuccess)
    return e;
  return allow_dynamic_lds((const void*)stream_bneck_kernel<K, true>, K::LDS_BYTES, lds_allowed[1]);
}

// Byte offsets from x are 32-bit inside the kernel.
template <class K>
constexpr size_t stream_max_map_bytes() { return (size_t)1 << 31; }

template <class K>
hipError_t launch_stream(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                         const void* packed, const float* b1, const float* b2, const float* b3,
                         void* out, bool post_relu, hipStream_t st) {
  if ((size_t)g.N * g.H * g.W * K::C * 2 > stream_max_map_bytes<K>()) return hipErrorInvalidValue;
  auto k = post_relu ? stream_bneck_kernel<K, true> : stream_bneck_kernel<K, false>;
  if (hipError_t e = prepare_stream<K>(); e != hipSuccess) return e;
  // one persistent workgroup per CU; more only when a run would exceed what a workgroup stages
  int grid = device_cu_count();
  const int need = (g.P + K::MAXQ - 1) / K::MAXQ;
  if (grid < need) grid = need;
  if (grid > g.P) grid = g.P;
  const __bf16* p1 = (const __bf16*)packed;
  const __bf16* p2 = p1 + (size_t)K::M * K::C;
  const __bf16* p3 = p2 + 9 * (size_t)K::M * K::M;
  hipLaunchKernelGGL(k, dim3(grid), dim3(K::NT), K::LDS_BYTES, st, g, (const __bf16*)x, idx, count, p1, b1,
                     p2, b2, p3, b3, (__bf16*)out);
  return hipGetLastError();
}

}  // namespace
}  // namespace lasnet
