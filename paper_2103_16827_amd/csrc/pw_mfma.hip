// Pointwise (k = 1) int8 convolution = GEMM  Y[t, co] = sum_ci X[ci, t] * W[co, ci]  on the
// gfx950 int8 matrix cores, with the fused epilogue (bias, dyadic rescale, residual, clamp).
//
// The activation layout [C, T] has frames contiguous, the contraction runs over channels.  This
// kernel copies each [64 channels][TM frames] chunk of the tile into LDS unchanged (16-byte
// loads and stores along the frame axis) and lets the LDS transpose read (ds_read_b64_tr_b8)
// deliver the MFMA operand: within 16 lanes, lane i receives byte (i & 7) of the 8-byte row
// addressed by lane 2j + (i >> 3) as its byte j, i.e. a column of an 8 x 16 byte block.  With
// lane l of a 16-lane group addressing channel row (l >> 1), frames 8 (l & 1)..+8, lane m ends up
// with 8 consecutive channels of frame m - the A operand (rows = frames, K = channels) of
// v_mfma_i32_16x16x64_i8.  The order of K inside an operand is free as long as both operands
// agree: lane group gi takes channels 8 gi..+8 and 32 + 8 gi..+8 of the chunk, so that one
// transpose read of the four lane groups covers 32 consecutive channel rows; the packed weight
// layout stores the B operand in exactly that order (plain weights are fetched as the two
// matching 8-byte pieces).  LDS row pitch = 16 * odd >= TM bytes: 16 consecutive channel rows
// then hit distinct banks.
//
// Memory latency is hidden by a register-staged pipeline three chunks deep: while chunk kc is
// multiplied out of LDS, the global loads of chunks kc+1..kc+3 (activations and weights) are in
// flight.  The loop is unrolled four times so that every buffer index is a compile-time constant,
// and every global load is unconditional (addresses are clamped instead of predicated; frames past
// the end of a row only feed output frames that are never stored), so that the number of loads in
// flight at each wait is known statically and a wait never drains the younger prefetches.  This
// needs Cin to be a multiple of 256.
#include "kernels.hpp"

#include <cstdio>
#include <cstdlib>

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

template <int MT, int NT, bool PACKED>
__global__ __launch_bounds__(256) void pw_mfma_kernel(ConvParams p, PwGeom g) {
  constexpr int TM = 16 * MT, TN = 64 * NT;
  constexpr int Q = TM / 16;                                  // 16-byte units per row
  constexpr int RS = 16 * (Q | 1);                            // row pitch: 16 * odd >= TM
  constexpr int UNITS = 64 * Q;                               // 16-byte units per chunk
  constexpr int ROUNDS = (UNITS + 255) / 256;
  constexpr int DEPTH = 4;                                    // register stages (3 chunks ahead)
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
  const int kch = g.kchunks;

  // ---- per-thread copy plan: unit u = tid + 256 it -> (row r, 16-byte column q)
  // Threads past the end of the chunk and columns past the end of the row re-read a valid unit.
  const int8_t* xsrc[ROUNDS];
  int xdst[ROUNDS];
#pragma unroll
  for (int it = 0; it < ROUNDS; ++it) {
    const int u = min(tid + 256 * it, UNITS - 1);
    const int r = u / Q, q = u - r * Q;
    const int tq = min(t0 + 16 * q, p.Tin - 16);
    xsrc[it] = p.x + (int64_t)b * p.xbs + (int64_t)r * p.Tin + tq;
    xdst[it] = r * RS + 16 * q;
  }
  const int64_t xstep = (int64_t)64 * p.Tin;                  // one chunk further down the channels

  // ---- per-lane weight stream: block (co16, kc) of the packed layout, or plain rows
  const int8_t* wsrc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (PACKED) {
      const int co16 = min((co_w >> 4) + nt, ((p.Cout + 15) >> 4) - 1);
      wsrc[nt] = p.w + ((int64_t)co16 * kch * 64 + lane) * 16;
    } else {
      wsrc[nt] = p.w + (int64_t)min(co_w + 16 * nt + n, p.Cout - 1) * p.Cin + 8 * gi;
    }
  }

  v4i xst[DEPTH][ROUNDS];
  v4i wst[DEPTH][NT];
  auto issue = [&](int kc, int slot) {
#pragma unroll
    for (int it = 0; it < ROUNDS; ++it)
      xst[slot][it] = *reinterpret_cast<const v4i*>(xsrc[it] + kc * xstep);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      if (PACKED) {
        wst[slot][nt] = *reinterpret_cast<const v4i*>(wsrc[nt] + (int64_t)kc * 1024);
      } else {
        const v2i w0 = *reinterpret_cast<const v2i*>(wsrc[nt] + 64 * kc);
        const v2i w1 = *reinterpret_cast<const v2i*>(wsrc[nt] + 64 * kc + 32);
        wst[slot][nt] = (v4i){w0.x, w0.y, w1.x, w1.y};
      }
    }
  };
  auto to_lds = [&](int slot, int buf) {
#pragma unroll
    for (int it = 0; it < ROUNDS; ++it)
      if (tid + 256 * it < UNITS) *reinterpret_cast<v4i*>(&xs[buf][xdst[it]]) = xst[slot][it];
  };

  // ---- per-channel constants first (oldest loads in flight); accumulators start at the bias
  v4i acc[MT][NT];
  int32_t mc[NT], sc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int co = min(co_w + 16 * nt + n, p.Cout - 1);
    const int32_t bv = p.bias ? p.bias[co] : 0;
    mc[nt] = p.m[co];
    sc[nt] = p.s[co];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = (v4i){bv, bv, bv, bv};
  }

  // transpose-read address of this lane inside a chunk buffer (row pair / half, see header)
  const int l16 = lane & 15;
  const int tr_off = (8 * gi + (l16 >> 1)) * RS + 8 * (l16 & 1);

  auto multiply = [&](int ph) {
    const unsigned char* base = &xs[ph & 1][tr_off];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const v2i a0 = lds_read_tr8(base + 16 * mt);
      const v2i a1 = lds_read_tr8(base + 32 * RS + 16 * mt);
      const v4i a = {a0.x, a0.y, a1.x, a1.y};
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, wst[ph][nt], acc[mt][nt], 0, 0, 0);
    }
  };

  issue(0, 0);
  issue(1, 1);
  issue(2, 2);
  to_lds(0, 0);
  __syncthreads();

  // steady state: chunk kc0 + ph is multiplied while chunk kc0 + ph + 3 is requested
  int kc0 = 0;
  for (; kc0 + DEPTH < kch; kc0 += DEPTH) {
#pragma unroll
    for (int ph = 0; ph < DEPTH; ++ph) {
      issue(kc0 + ph + 3, (ph + 3) % DEPTH);
      multiply(ph);
      to_lds((ph + 1) % DEPTH, (ph + 1) & 1);
      __syncthreads();
    }
  }
  // last four chunks: only the first still has a chunk to request
  issue(kc0 + 3, 3);
#pragma unroll
  for (int ph = 0; ph < DEPTH; ++ph) {
    multiply(ph);
    if (ph + 1 < DEPTH) {
      to_lds(ph + 1, (ph + 1) & 1);
      __syncthreads();
    }
  }

  // ---- epilogue: lane (n, gi) holds frames t0 + 16 mt + 4 gi + (0..3) of channel co_w + 16 nt + n
  const int lo = p.relu ? 0 : -128;
  bool fast = true;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) fast = fast && sc[nt] >= 33;
  const bool all_fast = __all(fast);                          // wave-uniform: one code path
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int co = co_w + 16 * nt + n;
    if (co >= p.Cout) continue;
    const int64_t orow = (int64_t)b * p.ybs + (int64_t)co * p.Tout + t0 + 4 * gi;
    int8_t* yrow = p.y + orow;
    const int8_t* rrow = p.res ? p.res + orow : nullptr;
    const int sh = sc[nt] - 32, rnd = all_fast ? 1 << (sc[nt] - 33) : 0;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if (t0 + 16 * mt + 4 * gi >= p.Tout) continue;
      int32_t v[4];
      if (all_fast) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = ((int32_t)__mulhi(acc[mt][nt][i], mc[nt]) + rnd) >> sh;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = dyadic_rescale(acc[mt][nt][i], mc[nt], sc[nt]);
      }
      if (rrow) {
        const uint32_t rw = *reinterpret_cast<const uint32_t*>(rrow + 16 * mt);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] += (int32_t)(int8_t)(rw >> (8 * i));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = clamp_i8(v[i], lo);
      const uint32_t p01 = __builtin_amdgcn_perm((uint32_t)v[1], (uint32_t)v[0], 0x0c0c0400u);
      const uint32_t p23 = __builtin_amdgcn_perm((uint32_t)v[3], (uint32_t)v[2], 0x04000c0cu);
      *reinterpret_cast<uint32_t*>(yrow + 16 * mt) = p01 | p23;
    }
  }
}

struct Choice { int MT, NT; };

bool pick(const ConvParams& p, Choice& c) {
  static const int MTs[] = {2, 5, 8, 10}, NTs[] = {1, 2, 4};
  if (const char* e = getenv("QASR_PW_TILE")) {          // tuning override: "MT,NT"
    int mt = 0, nt = 0;
    if (sscanf(e, "%d,%d", &mt, &nt) == 2)
      for (int MT : MTs)
        for (int NT : NTs)
          if (MT == mt && NT == nt) { c.MT = mt; c.NT = nt; return true; }
  }
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
  if (p.w_packed)
    return launch_kernel(pw_mfma_kernel<MT, NT, true>, dim3((unsigned)blocks), dim3(256), 0, st, p, g);
  return launch_kernel(pw_mfma_kernel<MT, NT, false>, dim3((unsigned)blocks), dim3(256), 0, st, p, g);
}

}  // namespace

bool pw_mfma_supported(const ConvParams& p) {
  if (p.depthwise || p.k != 1 || p.stride != 1 || p.pl != 0 || p.Tout != p.Tin) return false;
  if (p.Cin % 256 != 0 || p.Tin % 16 != 0 || p.xbs % 16 != 0 || p.ybs % 4 != 0) return false;
  if ((uintptr_t)p.x % 16 || (uintptr_t)p.y % 4 || (uintptr_t)p.w % 16 || (p.res && (uintptr_t)p.res % 4))
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
