// Dense int8 convolution (k >= 2 taps, any stride / dilation) as an implicit GEMM on the gfx950
// int8 matrix cores (v_mfma_i32_16x16x64_i8), software-pipelined over the contraction, with the
// fused epilogue (bias, dyadic rescale, residual, clamp).
//
//     Y[t, co] = sum_j sum_ci X[ci, t*stride - pad_left + j*dilation] * W[j][co][ci]
//
// Roles and layouts are those of gemm_mfma.hip: the A operand is the activation tile transposed
// (rows = output frames, K = input channels), the B operand the weight tile (packed form: 1 KiB
// contiguous per wave-wide load); a workgroup of 4 waves owns 16 MT output frames of one batch
// item and 256 output channels (64 per wave); each 64-channel chunk of the tile (with the time
// halo the taps need) is transposed in registers (4x4 byte blocks, v_perm_b32) into LDS rows
// [frame][64 channels], 80-byte pitch, so that a tap is a row offset.
//
// What differs is the order in time.  gemm_mfma loads and transposes a chunk, synchronises,
// multiplies its k taps, synchronises: the memory latency of every chunk and the L2 latency of
// every tap's weights are exposed.  Here the contraction is one flat stream of (chunk, tap) steps:
//   - the weights of step q + 2 are requested while step q is multiplied (ring of three);
//   - the global loads of chunk c + 1 are issued when chunk c starts, their transposition and LDS
//     writes (into the other of two LDS buffers) happen in the middle of chunk c's taps, under
//     the matrix products; one barrier per chunk, at its end.
// Every wave still streams its own weights from L2 (1 KiB per MT products), which is what bounds
// the big layers: staging the weights of a step in LDS for all waves would be the next step.
#include "kernels.hpp"

#include <cstdlib>

namespace qasr {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kXS = 80;       // LDS row pitch in bytes: 64 channels + 16 pad
constexpr int NT = 4;         // 16-channel columns per wave
constexpr int NBLK = 6;       // 4x4 blocks per thread and chunk at most: rows <= 384

struct CpGeom {
  int n_tt, n_co;     // frame tiles per batch item, channel tiles
  int rows;           // LDS rows (input frames incl. halo, rounded to 4)
  int kchunks;        // Cin / 64
  int co16n;          // ceil(Cout / 16)
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

template <int MT>
__global__ __launch_bounds__(256) void conv_pipe_kernel(ConvParams p, CpGeom g) {
  extern __shared__ __align__(16) unsigned char xs[];   // [2 buffers][rows][kXS]
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
  const int bufbytes = g.rows * kXS;

  const int8_t* xb = p.x + (int64_t)b * p.xbs;

  // ---- activation chunk kc: global -> registers (issue), registers -> LDS transposed (commit).
  // Thread-owned 4x4 blocks: block index blk = tid + 256 i covers frames 4 fq..+4 of channels
  // 4 cq..+4 of the chunk.
  const int nfq = g.rows >> 2;                      // frame quads per chunk
  const int nblk = 16 * nfq;                        // 4x4 blocks per chunk
  uint32_t xr[NBLK][4];
  auto issue_chunk = [&](int kc) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      const int blk = tid + 256 * i;
      const int fq = blk % nfq, cq = blk / nfq;
      const int f = fa + 4 * fq;
#pragma unroll
      for (int e = 0; e < 4; ++e) xr[i][e] = 0;
      if (blk < nblk && f >= 0 && f < p.Tin) {
        const int8_t* src = xb + (int64_t)(64 * kc + 4 * cq) * p.Tin + f;
#pragma unroll
        for (int e = 0; e < 4; ++e) xr[i][e] = *reinterpret_cast<const uint32_t*>(src + (int64_t)e * p.Tin);
      }
    }
  };
  auto commit_chunk = [&](int buf) __attribute__((always_inline)) {
    unsigned char* dst = xs + buf * bufbytes;
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      const int blk = tid + 256 * i;
      if (blk < nblk) {
        const int fq = blk % nfq, cq = blk / nfq;
        uint32_t c[4];
        transpose4x4(xr[i][0], xr[i][1], xr[i][2], xr[i][3], c);
        // channels 4 cq..+4 go to the column that the operand order assigns them
        const int col = 16 * ((cq >> 1) & 3) + 8 * (cq >> 3) + 4 * (cq & 1);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          *reinterpret_cast<uint32_t*>(dst + (4 * fq + e) * kXS + col) = c[e];
      }
    }
  };

  // ---- weights: step q = (chunk, tap) of the flat contraction, ring of three steps
  const int Q = g.kchunks * p.k;
  int wkc = 0, wj = 0;                              // chunk and tap of the next step to request
  auto load_w = [&](v4i (&dst)[NT]) __attribute__((always_inline)) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int co16 = min((co_w >> 4) + nt, g.co16n - 1);
      dst[nt] = *reinterpret_cast<const v4i*>(
          p.w + ((((int64_t)wj * g.co16n + co16) * g.kchunks + wkc) * 64 + lane) * 16);
    }
    if (wkc * p.k + wj < Q - 1) {                   // (the stream stays on its last step at the end)
      if (++wj == p.k) { wj = 0; ++wkc; }
    }
  };

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

  // ---- prologue: chunk 0 into buffer 0, weights of steps 0 and 1
  v4i wb[3][NT];
  issue_chunk(0);
  load_w(wb[0]);
  load_w(wb[1]);
  commit_chunk(0);
  __syncthreads();

  const int jmid = p.k >> 1;                        // the tap at which the next chunk is committed
  int kc = 0, j = 0;                                // chunk and tap of the current step
  if (g.kchunks > 1) issue_chunk(1);
  for (int q = 0; q < Q; q += 3) {
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      if (q + u < Q) {
        load_w(wb[(u + 2) % 3]);
        const unsigned char* arow = xs + (kc & 1) * bufbytes + (foff + j * p.dil + n * p.stride) * kXS + 16 * gi;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const v4i a = *reinterpret_cast<const v4i*>(arow + 16 * mt * p.stride * kXS);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, wb[u][nt], acc[mt][nt], 0, 0, 0);
        }
        if (j == jmid && kc + 1 < g.kchunks) commit_chunk((kc + 1) & 1);
        if (++j == p.k) {
          j = 0;
          ++kc;
          __syncthreads();                          // chunk kc is in LDS; chunk kc - 1 has been read by all
          if (kc + 1 < g.kchunks) issue_chunk(kc + 1);
        }
      }
    }
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

int lds_rows(const ConvParams& p, int TM) {
  // frames read by a tile: (TM-1)*stride + dil*(k-1) + 1, plus up to 3 of dword alignment slack
  return (((TM - 1) * p.stride + p.dil * (p.k - 1) + 1 + 3) + 3) & ~3;
}

bool pick(const ConvParams& p, int& MT) {
  if (getenv("QASR_NO_CONV_PIPE")) return false;          // tuning: fall through to gemm_mfma
  if (p.depthwise || p.Cin % 64 != 0 || !p.w_packed || p.k < 2) return false;
  if (p.Cout < 64) return false;
  if (p.Tin % 4 != 0 || p.Tout % 4 != 0 || p.xbs % 4 != 0 || p.ybs % 4 != 0) return false;
  if ((uintptr_t)p.x % 4 || (uintptr_t)p.y % 4 || (uintptr_t)p.w % 16 || (p.res && (uintptr_t)p.res % 4))
    return false;
  // frames per tile: 96 or 64 (128 would need all 256 registers and leave one wave per SIMD:
  // measured slower than 96 with two)
  static const int MTs[] = {6, 4};
  double best = 1e300;
  bool found = false;
  for (int mt : MTs) {
    const int TM = 16 * mt;
    const int rows = lds_rows(p, TM);
    if (rows > 64 * NBLK || (int64_t)2 * rows * kXS > 64 * 1024) continue;
    const int64_t n_tt = (p.Tout + TM - 1) / TM, n_co = (p.Cout + 64 * NT - 1) / (64 * NT);
    const int64_t blocks = (int64_t)p.B * n_tt * n_co;
    if (blocks > 0x7fffffffLL) continue;
    // frames computed per useful frame (tile round-up) and halo read per tile
    const double cost = (double)(n_tt * TM) / (double)p.Tout * (1.0 + 2.0 / mt);
    if (cost < best) { best = cost; MT = mt; found = true; }
  }
  return found;
}

template <int MT>
hipError_t launch_t(const ConvParams& p, hipStream_t st) {
  constexpr int TM = 16 * MT, TN = 64 * NT;
  CpGeom g;
  g.n_tt = (p.Tout + TM - 1) / TM;
  g.n_co = (p.Cout + TN - 1) / TN;
  g.rows = lds_rows(p, TM);
  g.kchunks = p.Cin / 64;
  g.co16n = (p.Cout + 15) / 16;
  const int64_t blocks = (int64_t)p.B * g.n_tt * g.n_co;
  return launch_kernel(conv_pipe_kernel<MT>, dim3((unsigned)blocks), dim3(256),
                       (size_t)2 * g.rows * kXS, st, p, g);
}

}  // namespace

bool conv_pipe_supported(const ConvParams& p) {
  int MT;
  return pick(p, MT);
}

hipError_t launch_conv_pipe(const ConvParams& p, hipStream_t st) {
  int MT;
  if (!pick(p, MT)) return hipErrorInvalidValue;
  if (MT == 6) return launch_t<6>(p, st);
  return launch_t<4>(p, st);
}

}  // namespace qasr
