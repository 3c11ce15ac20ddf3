// Pointwise (k = 1) int8 convolution = GEMM  Y[t, co] = sum_ci X[ci, t] * W[co, ci]  on the
// gfx950 int8 matrix cores, with the fused epilogue (bias, dyadic rescale, residual, clamp).
//
// The activation layout [C, T] has frames contiguous, the contraction runs over channels.  This
// kernel copies each [64 channels][TM frames] chunk of the tile into LDS unchanged (16-byte
// loads and stores along the frame axis, double-buffered) and lets the LDS transpose read
// (ds_read_b64_tr_b8) deliver the MFMA operand: within 16 lanes, lane i receives byte (i & 7) of
// the 8-byte row addressed by lane 2j + (i >> 3) as its byte j, i.e. a column of an 8 x 16 byte
// block.  With lane l of a 16-lane group addressing channel row (l >> 1), frames 8 (l & 1)..+8,
// lane m ends up with 8 consecutive channels of frame m - the A operand (rows = frames,
// K = channels) of v_mfma_i32_16x16x64_i8.  The order of K inside an operand is free as long as
// both operands agree: lane group gi takes channels 8 gi..+8 and 32 + 8 gi..+8 of the chunk, so
// that one transpose read of the four lane groups covers 32 consecutive channel rows, and the
// weight operand is loaded from global memory / L2 as the matching two 8-byte pieces.
// LDS row pitch = 16 * odd >= TM bytes: 16 consecutive channel rows then hit distinct banks.
#include "kernels.hpp"

namespace qasr {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

namespace {

struct PwGeom {
  int n_tt, n_co, kchunks;
};

__device__ __forceinline__ v2i lds_read_tr8(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr8_b64_v2i32(
      (v2i __attribute__((address_space(3)))*)(const_cast<unsigned char*>(p)));
}

template <int MT, int NT>
__global__ __launch_bounds__(256) void pw_mfma_kernel(ConvParams p, PwGeom g) {
  constexpr int TM = 16 * MT, TN = 64 * NT;
  constexpr int Q = TM / 16;                                  // 16-byte units per row
  constexpr int RS = 16 * (Q | 1);                            // row pitch: 16 * odd >= TM
  constexpr int UNITS = 64 * Q;                               // 16-byte units per chunk
  constexpr int ROUNDS = (UNITS + 255) / 256;
  __shared__ __align__(16) unsigned char xs[2][64 * RS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, gi = lane >> 4;

  int id = blockIdx.x;
  const int co_tile = id % g.n_co;
  id /= g.n_co;
  const int t_tile = id % g.n_tt;
  const int b = id / g.n_tt;
  const int t0 = t_tile * TM;
  const int co_w = co_tile * TN + wave * 16 * NT;
  const int8_t* xb = p.x + (int64_t)b * p.xbs + t0;

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

  // copy plan of this thread: unit u = tid + 256 it -> (row r, 16-byte column q)
  int4 stage[ROUNDS];
  auto load_chunk = [&](int kc) {
#pragma unroll
    for (int it = 0; it < ROUNDS; ++it) {
      const int u = tid + 256 * it;
      const int r = u / Q, q = u - r * Q;
      stage[it] = make_int4(0, 0, 0, 0);
      if (u < UNITS && t0 + 16 * q < p.Tin)
        stage[it] = *reinterpret_cast<const int4*>(xb + (int64_t)(64 * kc + r) * p.Tin + 16 * q);
    }
  };
  auto store_chunk = [&](int buf) {
#pragma unroll
    for (int it = 0; it < ROUNDS; ++it) {
      const int u = tid + 256 * it;
      const int r = u / Q, q = u - r * Q;
      if (u < UNITS) *reinterpret_cast<int4*>(&xs[buf][r * RS + 16 * q]) = stage[it];
    }
  };
  v2i wreg[2][NT][2];
  auto load_w = [&](int kc, int slot) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int8_t* wp = p.w + (int64_t)co_ld[nt] * p.Cin + 64 * kc + 8 * gi;
      wreg[slot][nt][0] = *reinterpret_cast<const v2i*>(wp);
      wreg[slot][nt][1] = *reinterpret_cast<const v2i*>(wp + 32);
    }
  };

  load_chunk(0);
  load_w(0, 0);
  store_chunk(0);
  __syncthreads();

  // transpose-read address of this lane inside a chunk buffer (row pair / half, see header)
  const int l16 = lane & 15;
  const int tr_off = (8 * gi + (l16 >> 1)) * RS + 8 * (l16 & 1);

  for (int kc = 0; kc < g.kchunks; ++kc) {
    const int cur = kc & 1;
    const bool more = kc + 1 < g.kchunks;
    if (more) {
      load_chunk(kc + 1);
      load_w(kc + 1, cur ^ 1);
    }
    const unsigned char* base = &xs[cur][tr_off];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const v2i a0 = lds_read_tr8(base + 16 * mt);
      const v2i a1 = lds_read_tr8(base + 32 * RS + 16 * mt);
      const v4i a = {a0.x, a0.y, a1.x, a1.y};
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const v4i w = {wreg[cur][nt][0].x, wreg[cur][nt][0].y, wreg[cur][nt][1].x, wreg[cur][nt][1].y};
        acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, w, acc[mt][nt], 0, 0, 0);
      }
    }
    if (more) store_chunk(cur ^ 1);
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
      if (t >= p.Tout) continue;
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

bool pick(const ConvParams& p, Choice& c) {
  static const int MTs[] = {2, 5, 8, 10}, NTs[] = {1, 2, 4};
  double best = 1e300;
  bool found = false;
  for (int MT : MTs)
    for (int NT : NTs) {
      const int TM = 16 * MT, TN = 64 * NT;
      const int64_t n_tt = (p.Tout + TM - 1) / TM, n_co = (p.Cout + TN - 1) / TN;
      const int64_t blocks = (int64_t)p.B * n_tt * n_co;
      if (blocks > 0x7fffffffLL) continue;
      const double rounds = (double)((blocks + 255) / 256);
      const double per_block = (double)TM * TN * (1.0 + 24.0 / (double)(MT * NT));
      const double cost = rounds * per_block;
      if (cost < best) { best = cost; c.MT = MT; c.NT = NT; found = true; }
    }
  return found;
}

template <int MT, int NT>
hipError_t launch_t(const ConvParams& p, hipStream_t st) {
  constexpr int TM = 16 * MT, TN = 64 * NT;
  PwGeom g;
  g.n_tt = (p.Tout + TM - 1) / TM;
  g.n_co = (p.Cout + TN - 1) / TN;
  g.kchunks = p.Cin / 64;
  const int64_t blocks = (int64_t)p.B * g.n_tt * g.n_co;
  return launch_kernel(pw_mfma_kernel<MT, NT>, dim3((unsigned)blocks), dim3(256), 0, st, p, g);
}

}  // namespace

bool pw_mfma_supported(const ConvParams& p) {
  if (p.depthwise || p.k != 1 || p.stride != 1 || p.pl != 0 || p.Tout != p.Tin) return false;
  if (p.Cin % 64 != 0 || p.Tin % 16 != 0 || p.xbs % 16 != 0 || p.ybs % 4 != 0) return false;
  if ((uintptr_t)p.x % 16 || (uintptr_t)p.y % 4 || (uintptr_t)p.w % 8 || (p.res && (uintptr_t)p.res % 4))
    return false;
  Choice c;
  return pick(p, c);
}

hipError_t launch_pw_mfma(const ConvParams& p, hipStream_t st) {
  Choice c;
  if (!pw_mfma_supported(p) || !pick(p, c)) return hipErrorInvalidValue;
#define QASR_CASE(M, N) if (c.MT == M && c.NT == N) return launch_t<M, N>(p, st);
  QASR_CASE(2, 1) QASR_CASE(2, 2) QASR_CASE(2, 4)
  QASR_CASE(5, 1) QASR_CASE(5, 2) QASR_CASE(5, 4)
  QASR_CASE(8, 1) QASR_CASE(8, 2) QASR_CASE(8, 4)
  QASR_CASE(10, 1) QASR_CASE(10, 2) QASR_CASE(10, 4)
#undef QASR_CASE
  return hipErrorInvalidValue;
}

}  // namespace qasr
