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
// Every wave streams its own weights from L2 (1 KiB per MT products); loading the same weights in
// all four waves (a timing experiment with wrong results) changed nothing, so that stream is not
// what bounds the kernel.  Small layers are bound by the number of workgroups instead: the tile
// (16 MT frames x 64 NT channels per wave) is chosen per layer by a small occupancy model.
#include "kernels.hpp"
#include "tuning.hpp"

#include <cmath>
#include <cstdio>
#include <cstdlib>

namespace qasr {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kXS = 80;       // LDS row pitch in bytes: 64 channels + 16 pad
constexpr int kMaxRows = 256; // one 4-frame x 16-channel unit per thread and chunk

struct CpGeom {
  int n_tt, n_co;     // frame tiles per batch item, channel tiles
  int rows;           // LDS rows (input frames incl. halo, rounded to 4)
  int kchunks;        // Cin / 64
  int co16n;          // ceil(Cout / 16)
  int tiles;          // B * n_tt * n_co
  int per_xcd;        // ceil(tiles / 8): tiles of one XCD (the grid is 8 * per_xcd workgroups)
};

template <int MT, int NT>
__global__ __launch_bounds__(256) void conv_pipe_kernel(ConvParams p, CpGeom g) {
  extern __shared__ __align__(16) unsigned char xs[];   // [2 buffers][rows][kXS]
  constexpr int TM = 16 * MT, TN = 64 * NT;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, gi = lane >> 4;

  // Workgroup -> tile.  Consecutive workgroups go round-robin to the 8 XCDs, each with an L2 of its
  // own, and every workgroup streams the whole weight slice of its channel tile: so the tiles are
  // numbered channel tile first (slowest), then batch item, then frame tile, and XCD x takes the
  // contiguous run [x per_xcd, (x + 1) per_xcd) of that order.  An XCD then touches one channel tile,
  // two where its run crosses a boundary, instead of all of them, and its workgroups, which start
  // together and step through the same (chunk, tap) sequence, share each weight line while it is
  // in that L2; neighbouring frame tiles (shared halo lines) stay on one XCD as well.
  // (per_xcd == 0, a tuning override: the plain order, tile = workgroup index, for comparisons)
  const int v = g.per_xcd ? (int)(blockIdx.x & 7) * g.per_xcd + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  if (v >= g.tiles) return;                         // whole workgroup, before any barrier
  const int bt = v % (g.tiles / g.n_co);            // (b, t_tile) of the tile
  const int co_tile = v / (g.tiles / g.n_co);
  const int t_tile = bt % g.n_tt;
  const int b = bt / g.n_tt;

  const int t0 = t_tile * TM;                       // first output frame of the tile
  const int f0 = t0 * p.stride - p.pl;              // first input frame the tile reads
  const int fa = f0 & ~3;                           // rounded down to a dword (also if negative)
  const int foff = f0 - fa;
  const int co_w = co_tile * TN + wave * 16 * NT;   // first output channel of this wave
  const int bufbytes = g.rows * kXS;

  const int8_t* xb = p.x + (int64_t)b * p.xbs;

  // ---- activation chunk kc: global -> registers (issue), registers -> LDS transposed (commit).
  // A thread owns one unit of the chunk: frames 4 fq..+4 of the 16 channels that make one 16-byte
  // column group cg of the LDS rows (four 4x4 byte blocks, channel quads 2cg, 2cg+1, 2cg+8,
  // 2cg+9 in the operand order).  It writes four 16-byte rows; lanes with consecutive fq are
  // 320 bytes apart, which is 16 banks, so the four rows are written in an order rotated by
  // (fq >> 2) & 3: then 16 consecutive lanes cover all 64 banks.  The rotation costs nothing: it
  // is folded into the byte selectors of the first transposition stage.
  const int nfq = g.rows >> 2;                      // frame quads per chunk (<= 64)
  const int u_fq = tid % nfq, u_cg = tid / nfq;
  const int rot = (u_fq >> 2) & 3;
  const int u_f = fa + 4 * u_fq;                    // first input frame of the unit
  const bool u_on = u_cg < 4 && u_f >= 0 && u_f < p.Tin;
  const uint32_t xoff = u_on ? (uint32_t)(8 * u_cg * p.Tin + u_f) : 0u;   // (Cin Tin < 2^31)
  uint32_t sel_lo, sel_hi;                          // frames rot, rot+1 | rot+2, rot+3 of two rows
  {
    const uint32_t f0s = rot, f1s = (rot + 1) & 3, f2s = (rot + 2) & 3, f3s = (rot + 3) & 3;
    sel_lo = f0s | ((4 + f0s) << 8) | (f1s << 16) | ((4 + f1s) << 24);
    sel_hi = f2s | ((4 + f2s) << 8) | (f3s << 16) | ((4 + f3s) << 24);
  }
  uint32_t xr[4][4];
  auto issue_chunk = [&](int kc) __attribute__((always_inline)) {
    const int8_t* base = xb + (int64_t)(64 * kc) * p.Tin;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int c = 4 * ((i & 1) + 8 * (i >> 1)) + e;
        xr[i][e] = u_on ? *reinterpret_cast<const uint32_t*>(base + (int64_t)c * p.Tin + xoff) : 0u;
      }
  };
  auto commit_chunk = [&](int buf) __attribute__((always_inline)) {
    if (u_cg < 4) {
      unsigned char* dst = xs + buf * bufbytes + 4 * u_fq * kXS + 16 * u_cg;
      uint32_t c[4][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // r_e = 4 consecutive frames of channel e  ->  c_e = 4 consecutive channels of frame
        // (e + rot) & 3
        const uint32_t lo01 = __builtin_amdgcn_perm(xr[i][1], xr[i][0], sel_lo);
        const uint32_t hi01 = __builtin_amdgcn_perm(xr[i][1], xr[i][0], sel_hi);
        const uint32_t lo23 = __builtin_amdgcn_perm(xr[i][3], xr[i][2], sel_lo);
        const uint32_t hi23 = __builtin_amdgcn_perm(xr[i][3], xr[i][2], sel_hi);
        c[i][0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
        c[i][1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
        c[i][2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
        c[i][3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
        *reinterpret_cast<v4i*>(dst + ((e + rot) & 3) * kXS) =
            (v4i){(int)c[0][e], (int)c[1][e], (int)c[2][e], (int)c[3][e]};
    }
  };

  // ---- weights: step q = (chunk, tap) of the flat contraction, ring of three steps
  const int Q = g.kchunks * p.k;
  int wkc = 0, wj = 0;                              // chunk and tap of the next step to request
  // (the packed buffer is below 2 GiB: a wave-uniform base per step plus a 32-bit lane offset)
  uint32_t woff[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
    woff[nt] = (uint32_t)((min((co_w >> 4) + nt, g.co16n - 1) * g.kchunks * 64 + lane) * 16);
  auto load_w = [&](v4i (&dst)[NT]) __attribute__((always_inline)) {
    const int8_t* wbase = p.w + (int64_t)(wj * g.co16n * g.kchunks + wkc) * 1024;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) dst[nt] = *reinterpret_cast<const v4i*>(wbase + woff[nt]);
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

  // The A operands (one 16-byte LDS read per 16 frames) go through a ring of three registers,
  // two reads ahead of the products; the ring runs on across the steps of a chunk, so that a
  // step's first operands arrive under the previous step's products (a new chunk starts after
  // the barrier with two exposed reads).
  auto arow_of = [&](int kc_, int j_) __attribute__((always_inline)) {
    return xs + (kc_ & 1) * bufbytes + (foff + j_ * p.dil + n * p.stride) * kXS + 16 * gi;
  };
  auto read_a = [&](const unsigned char* arow, int mt) __attribute__((always_inline)) {
    return *reinterpret_cast<const v4i*>(arow + 16 * mt * p.stride * kXS);
  };
  const int jmid = p.k >> 1;                        // the tap at which the next chunk is committed
  int kc = 0, j = 0;                                // chunk and tap of the current step
  if (g.kchunks > 1) issue_chunk(1);
  v4i ar[3];
  ar[0] = read_a(arow_of(0, 0), 0);
  ar[1] = read_a(arow_of(0, 0), 1);
  for (int q = 0; q < Q; q += 3) {
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      if (q + u < Q) {
        load_w(wb[(u + 2) % 3]);
        const unsigned char* arow = arow_of(kc, j);
        const bool last_tap = j + 1 == p.k;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if (mt + 2 < MT) {
            ar[(u * MT + mt + 2) % 3] = read_a(arow, mt + 2);
          } else if (!last_tap) {
            ar[(u * MT + mt + 2) % 3] = read_a(arow + p.dil * kXS, mt + 2 - MT);
          }
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ar[(u * MT + mt) % 3], wb[u][nt], acc[mt][nt], 0, 0, 0);
        }
        if (j == jmid && kc + 1 < g.kchunks) commit_chunk((kc + 1) & 1);
        if (last_tap) {
          j = 0;
          ++kc;
          __syncthreads();                          // chunk kc is in LDS; chunk kc - 1 has been read by all
          if (kc + 1 < g.kchunks) issue_chunk(kc + 1);
          if (kc < g.kchunks) {
            ar[((u + 1) * MT) % 3] = read_a(arow_of(kc, 0), 0);
            ar[((u + 1) * MT + 1) % 3] = read_a(arow_of(kc, 0), 1);
          }
        } else {
          ++j;
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
      int32_t radd[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) radd[i] = (int32_t)(int8_t)(rr >> (8 * i));
#pragma unroll
      for (int r = 0; r < kMaxMoreRes; ++r)          // dense-residual layers: further operands
        if (r < p.n_res_more) {
          const uint32_t rw = *reinterpret_cast<const uint32_t*>(p.res_more[r] + orow + t);
#pragma unroll
          for (int i = 0; i < 4; ++i) radd[i] += (int32_t)(int8_t)(rw >> (8 * i));
        }
      uint32_t pk = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int32_t v = dyadic_rescale(acc[mt][nt][i], mc, sc) + radd[i];
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

// Cycles per (chunk, tap) step on the busiest compute unit, from a small model: a unit holds `occ`
// workgroups (one wave each per SIMD); a SIMD with w resident waves spends w M cycles in the matrix
// pipe per step (M = 16 MT NT), a lone wave cannot go below M plus its own latencies (operand reads,
// weight request, loop), and the operand reads of all waves share the unit's LDS port.
double step_cycles(int MT, int NT, int64_t blocks) {
  const int occ = NT == 4 ? 2 : MT > 4 ? 3 : 4;           // bound by registers
  // (a fourth bound: every wave streams its own NT KiB of weights per step out of L2; fitted, with
  // the lone wave's latency, to per-layer times of the Jasper shape under every forced tile: only
  // the widest layer, 768 -> 896 with k = 29, changes its tile, 250 -> 221 us)
  const double M = 16.0 * MT * NT, alone = M + 250.0, lds = 32.0 * MT, wstream = 80.0 * NT;
  auto T = [&](int64_t w) {
    return w == 0 ? 0.0 : fmax(fmax(fmax((double)w * M, alone), (double)w * lds), (double)w * wstream);
  };
  const int64_t n = (blocks + 255) / 256;                 // workgroups on the busiest unit
  return (double)(n / occ) * T(occ) + T(n % occ);
}

bool pick(const ConvParams& p, int& MT, int& NT) {
  if (tuning().no_conv_pipe) return false;                // tuning: fall through to gemm_mfma
  if (p.depthwise || p.Cin % 64 != 0 || !p.w_packed || p.k < 2) return false;
  if (p.Cout < 64) return false;
  if (p.Tin % 4 != 0 || p.Tout % 4 != 0 || p.xbs % 4 != 0 || p.ybs % 4 != 0) return false;
  if ((uintptr_t)p.x % 4 || (uintptr_t)p.y % 4 || (uintptr_t)p.w % 16 || (p.res && (uintptr_t)p.res % 4))
    return false;
  for (int r = 0; r < p.n_res_more; ++r)
    if ((uintptr_t)p.res_more[r] % 4) return false;
  // the kernel addresses the packed weights with 32-bit offsets
  if ((int64_t)p.k * ((p.Cout + 15) / 16) * (p.Cin / 64) * 1024 > 0x7fffffffLL) return false;
  // frames per tile: 96 or 64 (128 would need all 256 registers and leave one wave per SIMD:
  // measured slower than 96 with two); channels per tile: 256 or 128
  const int force_mt = tuning().cp_mt, force_nt = tuning().cp_nt;   // tuning
  static const int MTs[] = {8, 7, 6, 5, 4}, NTs[] = {4, 2};
  double best = 1e300;
  bool found = false;
  for (int nt : NTs)
    for (int mt : MTs) {
      if ((force_mt && mt != force_mt) || (force_nt && nt != force_nt)) continue;
      const int TM = 16 * mt;
      const int rows = lds_rows(p, TM);
      if (rows > kMaxRows || (int64_t)p.Cin * p.Tin > 0x7fffffffLL) continue;
      const int64_t n_tt = (p.Tout + TM - 1) / TM, n_co = (p.Cout + 64 * nt - 1) / (64 * nt);
      const int64_t blocks = (int64_t)p.B * n_tt * n_co;
      if (blocks > 0x7ffffff0LL) continue;
      // halo read and transposed per tile, relative to the products
      const double cost = step_cycles(mt, nt, blocks) * (1.0 + 0.25 / mt);
      if (cost < best * 0.999) { best = cost; MT = mt; NT = nt; found = true; }
    }
  return found;
}

template <int MT, int NT>
hipError_t launch_t(const ConvParams& p, hipStream_t st) {
  constexpr int TM = 16 * MT, TN = 64 * NT;
  CpGeom g;
  g.n_tt = (p.Tout + TM - 1) / TM;
  g.n_co = (p.Cout + TN - 1) / TN;
  g.rows = lds_rows(p, TM);
  g.kchunks = p.Cin / 64;
  g.co16n = (p.Cout + 15) / 16;
  const int64_t blocks = (int64_t)p.B * g.n_tt * g.n_co;
  g.tiles = (int)blocks;
  g.per_xcd = tuning().cp_plain_order ? 0 : (int)((blocks + 7) / 8);
  return launch_kernel(conv_pipe_kernel<MT, NT>, dim3((unsigned)(g.per_xcd ? 8 * g.per_xcd : (int)blocks)), dim3(256),
                       (size_t)2 * g.rows * kXS, st, p, g);
}

}  // namespace

bool conv_pipe_supported(const ConvParams& p) {
  int MT, NT;
  return pick(p, MT, NT);
}

hipError_t launch_conv_pipe(const ConvParams& p, hipStream_t st) {
  int MT, NT;
  if (!pick(p, MT, NT)) return hipErrorInvalidValue;
  switch (10 * MT + NT) {
    case 84: return launch_t<8, 4>(p, st);
    case 74: return launch_t<7, 4>(p, st);
    case 64: return launch_t<6, 4>(p, st);
    case 54: return launch_t<5, 4>(p, st);
    case 44: return launch_t<4, 4>(p, st);
    case 82: return launch_t<8, 2>(p, st);
    case 72: return launch_t<7, 2>(p, st);
    case 62: return launch_t<6, 2>(p, st);
    case 52: return launch_t<5, 2>(p, st);
    default: return launch_t<4, 2>(p, st);
  }
}

}  // namespace qasr
