// Pointwise and dense int8 convolution as an implicit GEMM on the gfx950 int8 matrix cores
// (v_mfma_i32_16x16x64_i8), with the fused epilogue (bias, dyadic rescale, residual, clamp).
//
//     Y[t, co] = sum_j sum_ci X[ci, t*stride - pad_left + j*dilation] * W[j][co][ci]
//
// MFMA roles: the A operand is the activation tile transposed (rows = output frames, K = input
// channels), the B operand is the weight tile (columns = output channels), so that an
// accumulator lane ends up with 4 consecutive frames of one output channel - the order in which
// [B, C, T] stores them.  A workgroup (4 waves) owns TM = 16*MT output frames of one batch item
// and TN = 64*NT output channels; all waves share the frame rows and split the channels.
//
// The activation layout [C, T] has frames contiguous but the contraction runs over channels, so
// each 64-channel chunk of the tile (with the time halo the taps need) is transposed on its way
// into LDS: 4x4 byte blocks are transposed in registers with v_perm_b32 and written as
// [frame][64 channels] rows (80-byte pitch, so that the 16-byte operand reads of 16 consecutive
// frames hit distinct banks).  A tap is then just a row offset; the transposition is paid once
// per chunk and amortised over the k taps.  Weights go straight from global memory / L2 to
// registers in operand layout (the packed form: 1 KiB contiguous per wave-wide load), prefetched
// one tap ahead.  The packed form orders the 64 channels of a chunk so that lane group gi holds
// channels 8 gi..+8 and 32 + 8 gi..+8; the LDS rows are written in the matching column order, so
// that an operand is still one 16-byte read.
#include "kernels.hpp"

namespace qasr {

typedef int v4i __attribute__((ext_vector_type(4)));

namespace {

constexpr int kXS = 80;   // LDS row pitch in bytes: 64 channels + 16 pad

struct GemmGeom {
  int n_tt, n_co;     // frame tiles per batch item, channel tiles
  int rows;           // LDS rows (input frames incl. halo, rounded to 4)
  int kchunks;        // Cin / 64
};

__device__ __forceinline__ void transpose4x4(uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3,
                                             uint32_t (&c)[4]) {
  // r_e = 4 consecutive frames of channel e  ->  c_f = 4 consecutive channels of frame f
  const uint32_t lo01 = __builtin_amdgcn_perm(r1, r0, 0x05010400u);
  const uint32_t hi01 = __builtin_amdgcn_perm(r1, r0, 0x07030602u);
  const uint32_t lo23 = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
  const uint32_t hi23 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
  c[0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
  c[1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
  c[2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
  c[3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
}

template <int MT, int NT>
__global__ __launch_bounds__(256) void gemm_conv_kernel(ConvParams p, GemmGeom g) {
  extern __shared__ __align__(16) unsigned char xs[];   // [rows][kXS]
  constexpr int TM = 16 * MT, TN = 64 * NT;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, gi = lane >> 4;

  int id = blockIdx.x;
  const int co_tile = id % g.n_co;
  id /= g.n_co;
  const int t_tile = id % g.n_tt;
  const int b = id / g.n_tt;

  const int t0 = t_tile * TM;                       // first output frame of the tile
  const int f0 = t0 * p.stride - p.pl;              // first input frame the tile reads
  const int fa = f0 & ~3;                           // rounded down to a dword (also if negative)
  const int foff = f0 - fa;
  const int co_w = co_tile * TN + wave * 16 * NT;   // first output channel of this wave

  const int8_t* xb = p.x + (int64_t)b * p.xbs;

  // per-lane output channels (clamped for reads; stores are masked)
  int co_ld[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) co_ld[nt] = min(co_w + 16 * nt + n, p.Cout - 1);

  v4i acc[MT][NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int32_t bv = p.bias ? p.bias[co_ld[nt]] : 0;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = (v4i){bv, bv, bv, bv};
  }

  const int nfq = g.rows >> 2;                      // frame quads per chunk
  const int nblk = 16 * nfq;                        // 4x4 blocks per chunk

  // weight operand of (tap j, chunk kc, column tile nt)
  const int co16n = (p.Cout + 15) >> 4;
  auto load_w = [&](int j, int kc, int nt) -> v4i {
    if (p.w_packed) {
      const int co16 = min((co_w >> 4) + nt, co16n - 1);
      return *reinterpret_cast<const v4i*>(
          p.w + ((((int64_t)j * co16n + co16) * g.kchunks + kc) * 64 + lane) * 16);
    }
    // plain [Cout][Cin] rows (k == 1 only): the two 8-byte pieces of the operand order
    const int8_t* wp = p.w + (int64_t)co_ld[nt] * p.Cin + 64 * kc + 8 * gi;
    const int2 w0 = *reinterpret_cast<const int2*>(wp);
    const int2 w1 = *reinterpret_cast<const int2*>(wp + 32);
    return (v4i){w0.x, w0.y, w1.x, w1.y};
  };

  for (int kc = 0; kc < g.kchunks; ++kc) {
    // ---- activation chunk: [64 ci][rows frames] -> LDS [frame][64 ci]
    for (int blk = tid; blk < nblk; blk += 256) {
      const int fq = blk % nfq, cq = blk / nfq;
      const int f = fa + 4 * fq;
      uint32_t r[4] = {0, 0, 0, 0};
      if (f >= 0 && f < p.Tin) {
        const int8_t* src = xb + (int64_t)(64 * kc + 4 * cq) * p.Tin + f;
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = *reinterpret_cast<const uint32_t*>(src + (int64_t)e * p.Tin);
      }
      uint32_t c[4];
      transpose4x4(r[0], r[1], r[2], r[3], c);
      // channels 4 cq..+4 go to the column that the operand order assigns them
      const int col = 16 * ((cq >> 1) & 3) + 8 * (cq >> 3) + 4 * (cq & 1);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        *reinterpret_cast<uint32_t*>(xs + (4 * fq + e) * kXS + col) = c[e];
    }
    __syncthreads();

    // ---- taps: weights one tap ahead in registers
    v4i wb[2][NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wb[0][nt] = load_w(0, kc, nt);
    for (int j = 0; j < p.k; j += 2) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int jj = j + half;
        if (jj < p.k) {
          if (jj + 1 < p.k) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) wb[half ^ 1][nt] = load_w(jj + 1, kc, nt);
          }
          const unsigned char* arow = xs + (foff + jj * p.dil + n * p.stride) * kXS + 16 * gi;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const v4i a = *reinterpret_cast<const v4i*>(arow + 16 * mt * p.stride * kXS);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, wb[half][nt], acc[mt][nt], 0, 0, 0);
          }
        }
      }
    }
    __syncthreads();
  }

  // ---- epilogue: lane (n, gi) holds frames t0 + 16 mt + 4 gi + (0..3) of channel co_w + 16 nt + n
  const int lo = p.relu ? 0 : -128;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int co = co_w + 16 * nt + n;
    if (co >= p.Cout) continue;
    const int32_t mc = p.m[co], sc = p.s[co];
    const int64_t orow = (int64_t)b * p.ybs + (int64_t)co * p.Tout;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int t = t0 + 16 * mt + 4 * gi;
      if (t >= p.Tout) continue;                    // Tout % 4 == 0: the whole dword is in or out
      uint32_t rr = 0;
      if (p.res) rr = *reinterpret_cast<const uint32_t*>(p.res + orow + t);
      uint32_t pk = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int32_t v = dyadic_rescale(acc[mt][nt][i], mc, sc) + (int32_t)(int8_t)(rr >> (8 * i));
        pk |= (uint32_t)(clamp_i8(v, lo) & 0xff) << (8 * i);
      }
      *reinterpret_cast<uint32_t*>(p.y + orow + t) = pk;
    }
  }
}

struct Choice { int MT, NT; };

int lds_rows(const ConvParams& p, int TM) {
  // frames read by a tile: (TM-1)*stride + dil*(k-1) + 1, plus up to 3 of dword alignment slack
  return (((TM - 1) * p.stride + p.dil * (p.k - 1) + 1 + 3) + 3) & ~3;
}

bool pick(const ConvParams& p, Choice& c) {
  static const int MTs[] = {2, 5, 8}, NTs[] = {1, 2, 4};
  double best = 1e300;
  bool found = false;
  for (int MT : MTs)
    for (int NT : NTs) {
      const int TM = 16 * MT, TN = 64 * NT;
      if ((int64_t)lds_rows(p, TM) * kXS > 64 * 1024) continue;
      const int64_t n_tt = (p.Tout + TM - 1) / TM, n_co = (p.Cout + TN - 1) / TN;
      const int64_t blocks = (int64_t)p.B * n_tt * n_co;
      if (blocks > 0x7fffffffLL) continue;
      // time model: rounds of 256 workgroups x (matrix work per tile + per-tile overhead)
      const double rounds = (double)((blocks + 255) / 256);
      const double per_block = (double)TM * TN * (1.0 + 24.0 / (double)(MT * NT)) ;
      const double cost = rounds * per_block;
      if (cost < best) { best = cost; c.MT = MT; c.NT = NT; found = true; }
    }
  return found;
}

template <int MT, int NT>
hipError_t launch_t(const ConvParams& p, hipStream_t st) {
  constexpr int TM = 16 * MT, TN = 64 * NT;
  GemmGeom g;
  g.n_tt = (p.Tout + TM - 1) / TM;
  g.n_co = (p.Cout + TN - 1) / TN;
  g.rows = lds_rows(p, TM);
  g.kchunks = p.Cin / 64;
  const int64_t blocks = (int64_t)p.B * g.n_tt * g.n_co;
  return launch_kernel(gemm_conv_kernel<MT, NT>, dim3((unsigned)blocks), dim3(256),
                       (size_t)g.rows * kXS, st, p, g);
}

}  // namespace

bool gemm_mfma_supported(const ConvParams& p) {
  if (p.depthwise || p.Cin % 64 != 0) return false;
  if (p.k > 1 && !p.w_packed) return false;
  if (p.Tin % 4 != 0 || p.Tout % 4 != 0 || p.xbs % 4 != 0 || p.ybs % 4 != 0) return false;
  if ((uintptr_t)p.x % 4 || (uintptr_t)p.y % 4 || (uintptr_t)p.w % 16 || (p.res && (uintptr_t)p.res % 4))
    return false;
  Choice c;
  return pick(p, c);
}

hipError_t launch_gemm_mfma(const ConvParams& p, hipStream_t st) {
  Choice c;
  if (!gemm_mfma_supported(p) || !pick(p, c)) return hipErrorInvalidValue;
#define QASR_CASE(M, N) if (c.MT == M && c.NT == N) return launch_t<M, N>(p, st);
  QASR_CASE(2, 1) QASR_CASE(2, 2) QASR_CASE(2, 4)
  QASR_CASE(5, 1) QASR_CASE(5, 2) QASR_CASE(5, 4)
  QASR_CASE(8, 1) QASR_CASE(8, 2) QASR_CASE(8, 4)
#undef QASR_CASE
  return hipErrorInvalidValue;
}

}  // namespace qasr
