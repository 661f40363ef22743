// Fused sparse bottleneck on the gfx950 matrix cores (bf16 in, fp32 accumulate).
//
// One workgroup owns PPW consecutive entries of the active-patch index list and runs the
// whole block for them without leaving the CU (Sec. 3.4 / App. B.1: gather fused into the
// dynamic convolution, scatter fused into the residual add; here all three convolutions
// are fused as well, so the packed patches never go back to memory):
//
//   phase 0  decode the cell ids into pixel indices of the (S+2)x(S+2) windows
//   phase 1  conv1: stream the gathered window rows of x through LDS in KC-channel
//            chunks (double buffered), y1 = ReLU(W1 x + b1) -> LDS, 0 outside the image
//   phase 2  conv2: implicit GEMM over the 9 taps reading y1 rows by window offset -> y2 LDS
//   phase 3  conv3 + b3 + residual x, rounded once, stored at the patch's position
//
// Every GEMM is computed transposed, D[channel][pixel] = W[channel][k] * act[pixel][k],
// with v_mfma_f32_16x16x32_bf16: the weight fragment (A operand) comes straight from
// global/L2 in the natural [out][in] layout (8 consecutive k per lane = one 16-byte load),
// the activation fragment (B operand) from LDS.  In the result a lane holds 4 consecutive
// rows = channels; the rows of the NB tiles of a pass are interleaved so that a lane ends
// up with 4*NB consecutive channels of one pixel, which makes the epilogues 8..32-byte
// vector accesses.  Waves are arranged WR x WC (pixel-blocks x channel-blocks) per phase.
#include "common.hpp"

namespace lasnet {
namespace {

__device__ inline floatx4 mfma16(bf16x8 a, bf16x8 b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

constexpr int cdiv(int a, int b) { return (a + b - 1) / b; }
constexpr int cmax(int a, int b) { return a > b ? a : b; }

template <int C_, int M_, int S_, int PPW_, int NW_, int KC_, int WR1_, int WC1_, int WR2_,
          int WC2_, int GS2_, int WR3_, int WC3_, int NB3_, int GS3_>
struct Cfg {
  static constexpr int C = C_, M = M_, S = S_, PPW = PPW_, NW = NW_, KC = KC_;
  static constexpr int NT = NW * 64;
  static constexpr int T = S + 2, WW = T * T;
  static constexpr int R1 = PPW * WW, R1B = cdiv(R1, 16), R1P = R1B * 16;
  static constexpr int R2 = PPW * S * S, R2B = cdiv(R2, 16), R2P = R2B * 16;
  static constexpr int LDX = KC + 8, LDY = M + 8;      // +16 bytes: rows land in distinct banks
  static constexpr int WR1 = WR1_, WC1 = WC1_, NBW1 = M / 16 / WC1, RBW1 = cdiv(R1B, WR1);
  static constexpr int WR2 = WR2_, WC2 = WC2_, NBW2 = M / 16 / WC2, RBW2 = cdiv(R2B, WR2);
  static constexpr int GS2 = GS2_;
  static constexpr int WR3 = WR3_, WC3 = WC3_, NBT3 = C / 16 / WC3, NB3 = NB3_, RBW3 = cdiv(R2B, WR3);
  static constexpr int GS3 = GS3_;
  static constexpr int MS = M / 32;                    // k-steps over the mid channels
  static constexpr int OFF_Y1 = ((R1P + R2P) * 4 + 15) / 16 * 16;
  static constexpr int Y1_BYTES = R1P * LDY * 2;
  static constexpr int OFF_XS = OFF_Y1 + Y1_BYTES;
  static constexpr int XS_BYTES = 2 * R1P * LDX * 2;
  static constexpr int Y2_BYTES = R2P * LDY * 2;
  static constexpr int LDS_BYTES = OFF_XS + cmax(XS_BYTES, Y2_BYTES);
  static_assert(WR1 * WC1 == NW && WR2 * WC2 == NW && WR3 * WC3 == NW, "wave grid");
  static_assert(M % (16 * WC1) == 0 && M % (16 * WC2) == 0 && C % (16 * WC3) == 0, "channel split");
  static_assert(NBT3 % NB3 == 0, "conv3 passes");
  static_assert(C % KC == 0 && KC % 32 == 0 && M % 32 == 0, "k steps");
  static_assert(MS % GS2 == 0 && MS % GS3 == 0, "weight groups stay inside one tap");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

// Channel held by A-operand row i (0..15) of tile j when NB tiles are interleaved.
__device__ inline int arow_channel(int base, int nb, int j, int i) {
  return base + (i >> 2) * (4 * nb) + j * 4 + (i & 3);
}

template <class K>
__global__ __launch_bounds__(K::NT) void fused_bneck_kernel(
    Geom g, const __bf16* __restrict__ x, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ count, const __bf16* __restrict__ W1,
    const float* __restrict__ b1, const __bf16* __restrict__ W2, const float* __restrict__ b2,
    const __bf16* __restrict__ W3, const float* __restrict__ b3, __bf16* __restrict__ out,
    int post_relu) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  int* rowpix = reinterpret_cast<int*>(smem);              // [R1P] pixel of conv1 row or -1
  int* pixq = rowpix + K::R1P;                             // [R2P] pixel of output row or -1
  __bf16* y1s = reinterpret_cast<__bf16*>(smem + K::OFF_Y1);
  __bf16* xs = reinterpret_cast<__bf16*>(smem + K::OFF_XS);
  __bf16* y2s = xs;                                        // xs is dead once conv1 is done

  constexpr int C = K::C, M = K::M, S = K::S, T = K::T, WW = K::WW;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int nact = idx ? min(*count, g.P) : g.P;
  const int first = blockIdx.x * K::PPW;
  if (first >= nact) return;                               // uniform over the workgroup

  // ---------------------------------------------------------------- phase 0
  for (int r = tid; r < K::R1P; r += K::NT) {
    int pix = -1;
    if (r < K::R1) {
      const int slot = r / WW, wp = r - slot * WW;
      const int e = first + slot;
      if (e < nact) {
        const int cell = idx ? idx[e] : e;
        const int n = cell / (g.G * g.GW), rem = cell - n * (g.G * g.GW);
        const int gy = rem / g.GW, gx = rem - gy * g.GW;
        const int h = gy * S + wp / T - 1, w = gx * S + wp % T - 1;
        if (h >= 0 && h < g.H && w >= 0 && w < g.W) pix = (n * g.H + h) * g.W + w;
      }
    }
    rowpix[r] = pix;
  }
  for (int q = tid; q < K::R2P; q += K::NT) {
    int pix = -1;
    if (q < K::R2) {
      const int slot = q / (S * S), r = q - slot * (S * S);
      const int e = first + slot;
      if (e < nact) {
        const int cell = idx ? idx[e] : e;
        const int n = cell / (g.G * g.GW), rem = cell - n * (g.G * g.GW);
        const int gy = rem / g.GW, gx = rem - gy * g.GW;
        pix = (n * g.H + gy * S + r / S) * g.W + gx * S + r % S;
      }
    }
    pixq[q] = pix;
  }
  __syncthreads();

  // ---------------------------------------------------------------- phase 1: conv1
  {
    constexpr int RBW = K::RBW1, NBW = K::NBW1, KS = K::KC / 32, NCH = C / K::KC;
    constexpr int SEGS = K::KC / 8, NPIECE = K::R1P * SEGS, NP = cdiv(NPIECE, K::NT);
    const int wr = wave / K::WC1, wc = wave % K::WC1;
    floatx4 acc[RBW][NBW];
#pragma unroll
    for (int i = 0; i < RBW; ++i)
#pragma unroll
      for (int j = 0; j < NBW; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    const __bf16* wrow[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
      wrow[j] = W1 + (size_t)arow_channel(wc * NBW * 16, NBW, j, l16) * C + 8 * lg;
    const __bf16* xsrc[NP];
    int xdst[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int piece = tid + p * K::NT;
      xsrc[p] = nullptr;
      xdst[p] = -1;
      if (piece < NPIECE) {
        const int row = piece / SEGS, seg = piece - row * SEGS;
        const int pix = rowpix[row];
        if (pix >= 0) xsrc[p] = x + (size_t)pix * C + seg * 8;
        xdst[p] = row * K::LDX + seg * 8;
      }
    }
    uint4 xr[NP];
    bf16x8 wa[KS][NBW], wb[KS][NBW];
    auto gload = [&](int ch) {
#pragma unroll
      for (int p = 0; p < NP; ++p)
        xr[p] = xsrc[p] ? *reinterpret_cast<const uint4*>(xsrc[p] + ch * K::KC) : uint4{0, 0, 0, 0};
    };
    auto sstore = [&](int buf) {
#pragma unroll
      for (int p = 0; p < NP; ++p)
        if (xdst[p] >= 0) *reinterpret_cast<uint4*>(xs + buf * (K::R1P * K::LDX) + xdst[p]) = xr[p];
    };
    auto wload = [&](bf16x8(&w)[KS][NBW], int ch) {
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int j = 0; j < NBW; ++j)
          w[s][j] = *reinterpret_cast<const bf16x8*>(wrow[j] + ch * K::KC + s * 32);
    };
    gload(0);
    wload(wa, 0);
    sstore(0);
    __syncthreads();
    for (int ch = 0; ch < NCH; ++ch) {
      const bool more = ch + 1 < NCH;
      if (more) {
        gload(ch + 1);
        wload(wb, ch + 1);
      }
      const __bf16* xb = xs + (ch & 1) * (K::R1P * K::LDX);
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int i = 0; i < RBW; ++i) {
          const int rb = wr + K::WR1 * i;
          if (rb < K::R1B) {
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(xb + (rb * 16 + l16) * K::LDX + s * 32 + 8 * lg);
#pragma unroll
            for (int j = 0; j < NBW; ++j) acc[i][j] = mfma16(wa[s][j], b, acc[i][j]);
          }
        }
      if (more) {
        sstore((ch + 1) & 1);
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
          for (int j = 0; j < NBW; ++j) wa[s][j] = wb[s][j];
      }
      __syncthreads();
    }
    // epilogue: + b1, ReLU, force 0 outside the image / on unused rows, round to bf16
    const int chb = wc * NBW * 16 + lg * 4 * NBW;
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
      const int rb = wr + K::WR1 * i;
      if (rb < K::R1B) {
        const int row = rb * 16 + l16;
        const bool valid = rowpix[row] >= 0;
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
          bf16x4 o;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float a = fmaxf(acc[i][j][v] + b1[chb + j * 4 + v], 0.f);
            o[v] = (__bf16)(valid ? a : 0.f);
          }
          *reinterpret_cast<bf16x4*>(y1s + row * K::LDY + chb + j * 4) = o;
        }
      }
    }
  }
  __syncthreads();

  // ---------------------------------------------------------------- phase 2: conv2 (3x3)
  {
    constexpr int RBW = K::RBW2, NBW = K::NBW2, GS = K::GS2, MS = K::MS;
    constexpr int GPT = MS / GS, NG = 9 * GPT;             // groups per tap, groups in all
    const int wr = wave / K::WC2, wc = wave % K::WC2;
    floatx4 acc[RBW][NBW];
#pragma unroll
    for (int i = 0; i < RBW; ++i)
#pragma unroll
      for (int j = 0; j < NBW; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    int brow[RBW];                                         // window row of tap (0,0)
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
      const int q = (wr + K::WR2 * i) * 16 + l16;
      brow[i] = 0;
      if (q < K::R2) {
        const int slot = q / (S * S), r = q - slot * (S * S);
        brow[i] = slot * WW + (r / S) * T + r % S;
      }
    }
    const __bf16* wrow[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
      wrow[j] = W2 + (size_t)arow_channel(wc * NBW * 16, NBW, j, l16) * (9 * M) + 8 * lg;
    bf16x8 wa[GS][NBW], wb[GS][NBW];
    auto wload = [&](bf16x8(&w)[GS][NBW], int grp) {
#pragma unroll
      for (int s = 0; s < GS; ++s)
#pragma unroll
        for (int j = 0; j < NBW; ++j)
          w[s][j] = *reinterpret_cast<const bf16x8*>(wrow[j] + (grp * GS + s) * 32);
    };
    wload(wa, 0);
    for (int grp = 0; grp < NG; ++grp) {
      if (grp + 1 < NG) wload(wb, grp + 1);
      const int tap = grp / GPT, m0 = (grp - tap * GPT) * GS * 32;
      const int toff = (tap / 3) * T + tap % 3;
#pragma unroll
      for (int s = 0; s < GS; ++s)
#pragma unroll
        for (int i = 0; i < RBW; ++i) {
          if (wr + K::WR2 * i < K::R2B) {
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(
                y1s + (brow[i] + toff) * K::LDY + m0 + s * 32 + 8 * lg);
#pragma unroll
            for (int j = 0; j < NBW; ++j) acc[i][j] = mfma16(wa[s][j], b, acc[i][j]);
          }
        }
      if (grp + 1 < NG) {
#pragma unroll
        for (int s = 0; s < GS; ++s)
#pragma unroll
          for (int j = 0; j < NBW; ++j) wa[s][j] = wb[s][j];
      }
    }
    const int chb = wc * NBW * 16 + lg * 4 * NBW;
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
      const int rb = wr + K::WR2 * i;
      if (rb < K::R2B) {
        const int q = rb * 16 + l16;
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
          bf16x4 o;
#pragma unroll
          for (int v = 0; v < 4; ++v) o[v] = (__bf16)fmaxf(acc[i][j][v] + b2[chb + j * 4 + v], 0.f);
          *reinterpret_cast<bf16x4*>(y2s + q * K::LDY + chb + j * 4) = o;
        }
      }
    }
  }
  __syncthreads();

  // ---------------------------------------------------------------- phase 3: conv3 + scatter-add
  {
    constexpr int RBW = K::RBW3, NB = K::NB3, GS = K::GS3, MS = K::MS, NG = MS / GS;
    constexpr int NPASS = K::NBT3 / NB;
    const int wr = wave / K::WC3, wc = wave % K::WC3;
    int pq[RBW];
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
      const int rb = wr + K::WR3 * i;
      pq[i] = rb < K::R2B ? pixq[rb * 16 + l16] : -1;
    }
    for (int pass = 0; pass < NPASS; ++pass) {
      const int cb0 = (wc * K::NBT3 + pass * NB) * 16;     // first channel of this pass
      floatx4 acc[RBW][NB];
#pragma unroll
      for (int i = 0; i < RBW; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
      const __bf16* wrow[NB];
#pragma unroll
      for (int j = 0; j < NB; ++j)
        wrow[j] = W3 + (size_t)arow_channel(cb0, NB, j, l16) * M + 8 * lg;
      bf16x8 wa[GS][NB], wb[GS][NB];
      auto wload = [&](bf16x8(&w)[GS][NB], int grp) {
#pragma unroll
        for (int s = 0; s < GS; ++s)
#pragma unroll
          for (int j = 0; j < NB; ++j)
            w[s][j] = *reinterpret_cast<const bf16x8*>(wrow[j] + (grp * GS + s) * 32);
      };
      wload(wa, 0);
#pragma unroll
      for (int grp = 0; grp < NG; ++grp) {
        if (grp + 1 < NG) wload(wb, grp + 1);
#pragma unroll
        for (int s = 0; s < GS; ++s)
#pragma unroll
          for (int i = 0; i < RBW; ++i) {
            const int rb = wr + K::WR3 * i;
            if (rb < K::R2B) {
              const bf16x8 b = *reinterpret_cast<const bf16x8*>(
                  y2s + (rb * 16 + l16) * K::LDY + (grp * GS + s) * 32 + 8 * lg);
#pragma unroll
              for (int j = 0; j < NB; ++j) acc[i][j] = mfma16(wa[s][j], b, acc[i][j]);
            }
          }
        if (grp + 1 < NG) {
#pragma unroll
          for (int s = 0; s < GS; ++s)
#pragma unroll
            for (int j = 0; j < NB; ++j) wa[s][j] = wb[s][j];
        }
      }
      // epilogue: residual add in fp32, one rounding, store at the patch's own pixels
      const int chb = cb0 + lg * 4 * NB;
#pragma unroll
      for (int i = 0; i < RBW; ++i) {
        if (pq[i] >= 0) {
          const size_t off = (size_t)pq[i] * C + chb;
#pragma unroll
          for (int j = 0; j < NB; ++j) {
            const bf16x4 xv = *reinterpret_cast<const bf16x4*>(x + off + j * 4);
            bf16x4 o;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              float r = (float)xv[v] + (acc[i][j][v] + b3[chb + j * 4 + v]);
              if (post_relu) r = fmaxf(r, 0.f);
              o[v] = (__bf16)r;
            }
            *reinterpret_cast<bf16x4*>(out + off + j * 4) = o;
          }
        }
      }
    }
  }
}

// ---- instantiations --------------------------------------------------------------
//            C     M   S PPW NW KC  conv1   conv2+GS   conv3 NB GS
using K_s3 = Cfg<1024, 256, 2, 8, 8, 64, 2, 4, 1, 8, 4, 1, 8, 4, 2>;   // ResNet-101 stage 3, S=2
using K_s3s7 = Cfg<1024, 256, 7, 1, 8, 64, 2, 4, 2, 4, 4, 2, 4, 4, 2>; // stage 3, S=7 (also the dense tile)
using K_s2 = Cfg<512, 128, 4, 4, 8, 64, 2, 4, 2, 4, 4, 2, 4, 4, 2>;    // stage 2, S=4
using K_s2s7 = Cfg<512, 128, 7, 2, 8, 64, 2, 4, 2, 4, 4, 2, 4, 4, 2>;  // stage 2, S=7 (dense tile)
using K_s1 = Cfg<256, 64, 8, 1, 8, 64, 4, 2, 4, 2, 2, 2, 4, 4, 2>;     // stage 1, S=8
using K_s1s4 = Cfg<256, 64, 4, 4, 8, 64, 4, 2, 4, 2, 2, 2, 4, 4, 2>;   // stage 1, S=4 (Table 1 block)
using K_s1s7 = Cfg<256, 64, 7, 2, 8, 64, 4, 2, 4, 2, 2, 2, 4, 4, 2>;   // stage 1, S=7 (dense tile)

template <class K>
hipError_t launch_one(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                      const BlockWeights& w, void* out, bool post_relu, hipStream_t st) {
  auto k = fused_bneck_kernel<K>;
  hipError_t e = hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     K::LDS_BYTES);
  if (e != hipSuccess) return e;
  const int grid = (g.P + K::PPW - 1) / K::PPW;
  hipLaunchKernelGGL(k, dim3(grid), dim3(K::NT), K::LDS_BYTES, st, g, (const __bf16*)x, idx, count,
                     (const __bf16*)w.W1, w.b1, (const __bf16*)w.W2, w.b2, (const __bf16*)w.W3,
                     w.b3, (__bf16*)out, (int)post_relu);
  return hipGetLastError();
}

}  // namespace

#define LASNET_FOR_EACH_MFMA_CFG(X) X(K_s3) X(K_s3s7) X(K_s2) X(K_s2s7) X(K_s1) X(K_s1s4) X(K_s1s7)

bool mfma_supported(int C, int M, int S) {
#define X(K) if (C == K::C && M == K::M && S == K::S) return true;
  LASNET_FOR_EACH_MFMA_CFG(X)
#undef X
  return false;
}

hipError_t launch_mfma(const Geom& g, const void* x, const int32_t* idx, const int32_t* count,
                       const BlockWeights& w, void* out, bool post_relu, hipStream_t st) {
  if (g.P == 0) return hipSuccess;
#define X(K) if (g.C == K::C && g.M == K::M && g.S == K::S) return launch_one<K>(g, x, idx, count, w, out, post_relu, st);
  LASNET_FOR_EACH_MFMA_CFG(X)
#undef X
  return hipErrorInvalidValue;
}

}  // namespace lasnet
