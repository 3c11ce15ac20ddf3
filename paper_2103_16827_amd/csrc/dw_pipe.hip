// Depthwise int8 convolution (stride 1) as a banded-Toeplitz product on the gfx950 int8 matrix
// cores, software-pipelined so that reads and writes of HBM overlap.
//
// The arithmetic is that of dw_mfma.hip:
//
//     Y[m, n] = sum_kappa A[m, kappa] * X[kappa, n]        (v_mfma_i32_16x16x64_i8)
//     output frame   t = T0 + 16 n + m                      (n: 16-frame group, m: frame in group)
//     X[kappa, n]    = x[o + 16 n + kappa],   o = T0 - pad_left - delta   (o is a multiple of 16)
//     A[m, kappa]    = w[j]  if kappa - m - delta == j * dilation, else 0
//
// What differs is the flow of data.  A kernel in which every wave loads its rows, computes and
// stores once runs as three chip-wide bursts (all loads, then all arithmetic, then all stores),
// and HBM sees only one direction at a time.  Here a workgroup owns one channel (one Toeplitz
// operand, built once) and each of its 4 waves walks through its share of the batch in iterations
// of R rows ("strips"): the rows of iteration i + 2 are requested before iteration i is computed
// and stored, so every wave always has reads and writes in flight.
//
// Requests are direct global->LDS loads into one of three per-wave row buffers (nothing that is
// still in flight ever lives in a register the compiler manages).  A lane's 16-byte chunk lies
// either inside the row or entirely in the implicit zero padding; padding chunks are zeroed once in
// all three buffers and their lanes are masked out of every load.  Rows past the end of the batch
// re-read the wave's last row (their outputs are rejected by the bounds of the output resource), so
// that every iteration issues the same number of requests.  Completion is waited for with explicit
// counts (vmem.hpp): a wave's requests complete in order, loads and stores alike, so before
// iteration i the wave allows exactly the requests issued after the loads of iteration i to stay
// outstanding:  loads(i+1), loads(i+2) [L each] + stores(i-2), stores(i-1) [one per 256-frame tile].
// Needs 16-byte aligned rows that are a multiple of 16 frames and at most ~1000 frames long,
// 4-byte aligned outputs and no residual operand; everything else is served by dw_mfma.hip.
#include "kernels.hpp"
#include "vmem.hpp"

#include <cstdio>
#include <cstdlib>
#include <type_traits>

namespace qasr {

namespace {

constexpr int kMaxTiles = 8; // 256-frame tiles per iteration: R * groups per strip <= 128

struct DwpGeom {
  int delta;      // (-pad_left) mod 16
  int PH;         // (pad_left + delta) / 16: left halo in 16-byte chunks
  int NCH;        // 16-byte chunks per strip buffer: groups + 4*KC - 1
  int G;          // 16-frame groups per row
  int tiles;      // 256-frame tiles per iteration: ceil(R * G / 16) <= kMaxTiles
  int spw;        // rows per wave (a multiple of R)
  int c_per_xcd;  // channels per XCD: ceil(C / 8)
  int dbg;        // tuning: 1 skip the tiles
};

template <int KC, int R, int NI>
__global__ __launch_bounds__(256) void dw_pipe_kernel(ConvParams p, DwpGeom g) {
  extern __shared__ __align__(16) unsigned char strips_lds[];      // [4 waves][3 buffers][R][NCH][16]
  __shared__ __align__(16) unsigned char a_lds[KC * 1024];         // A operand, register layout
  __shared__ unsigned char wrow[64 * KC + 16];                     // dilated, shifted weight row
  constexpr int L = R * NI;                                        // load requests per iteration

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Consecutive workgroups go round-robin to the 8 XCDs (one L2 each); rows of neighbouring
  // channels share a cache line where they meet, so each XCD takes a contiguous range of channels.
  const int c = (int)(blockIdx.x & 7) * g.c_per_xcd + (int)(blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= g.c_per_xcd || c >= p.Cout) return;   // whole workgroup
  const int n = lane & 15, gi = lane >> 4;
  unsigned char* const my = strips_lds + (size_t)wave * 3 * R * g.NCH * 16;     // 3 row buffers

  // rows (batch items) of this wave: [s_begin, s_end), R per iteration
  const int s_begin = min((int)(blockIdx.y * 4 + wave) * g.spw, p.B);
  const int s_end = min(s_begin + g.spw, p.B);
  const int n_it = (s_end - s_begin + R - 1) / R;

  // Requests of one iteration (always L of them): rows `row` .. `row + R - 1` into buffer `buf`.
  // Chunk u of a row holds frames 16 (u - PH) .. +15; lanes whose chunk is padding stay out.
  const int8_t* const xc = p.x + (int64_t)c * p.Tin;
  const int rowbytes = g.NCH * 16;
  bool lane_in[NI];
  int64_t lane_off[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int u = lane + 64 * ni, t = 16 * (u - g.PH);
    lane_in[ni] = u < g.NCH && t >= 0 && t < p.Tin;
    lane_off[ni] = t;
  }
  auto issue = [&](int row, int buf) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int8_t* src = xc + (int64_t)min(row + r, s_end - 1) * p.xbs;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        if (lane_in[ni]) direct_load16(src + lane_off[ni], my + (buf * R + r) * rowbytes + 1024 * ni);
    }
  };
  // padding chunks (and nothing else) are written here, once
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int u = lane + 64 * ni;
    if (u < g.NCH && !lane_in[ni])
      for (int q = 0; q < 3 * R; ++q) *reinterpret_cast<v4i*>(my + q * rowbytes + u * 16) = (v4i){0, 0, 0, 0};
  }
  if (s_begin < s_end) {          // (a wave without rows issues nothing and skips the loop below)
    issue(s_begin, 0);
    issue(s_begin + R, 1);
    issue(s_begin + 2 * R, 2);
  }

  // per-channel constants: uniform over the workgroup
  const int32_t bias = p.bias ? p.bias[c] : 0;
  const int32_t mc = p.m[c], sc = p.s[c];

  // ---- Toeplitz operand: wrow[q] = w[j] where q - 15 - delta == j * dilation
  for (int q = tid; q < 64 * KC + 16; q += 256) {
    const int rel = q - 15 - g.delta;
    int8_t v = 0;
    if (rel >= 0) {
      const int j = rel / p.dil;
      if (j * p.dil == rel && j < p.k) v = p.w[(int64_t)c * p.k + j];
    }
    wrow[q] = (unsigned char)v;
  }
  __syncthreads();
  {
    // A[m, kappa] = wrow[kappa - m + 15]; lane (m, gi) holds kappa = 64 kc + 16 gi + (0..15).
    const int al = tid >> 2, dwi = tid & 3;
    const int am = al & 15, ag = al >> 4;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int base = 64 * kc + 16 * ag + 4 * dwi - am + 15;
      const uint32_t v = (uint32_t)wrow[base] | ((uint32_t)wrow[base + 1] << 8) |
                         ((uint32_t)wrow[base + 2] << 16) | ((uint32_t)wrow[base + 3] << 24);
      reinterpret_cast<uint32_t*>(a_lds)[kc * 256 + tid] = v;
    }
  }
  __syncthreads();
  v4i a[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) a[kc] = *reinterpret_cast<const v4i*>(a_lds + kc * 1024 + lane * 16);

  const int lo = p.relu ? 0 : -128;
  const int32_t hi127 = 127;
  const bool fast = sc >= 33;                           // uniform: one channel per workgroup
  const int sh = fast ? sc - 32 : sc, rnd = fast ? 1 << (sc - 33) : 0;

  // The 16-frame groups of an iteration's R rows form one flat list of columns; tile j takes
  // columns 16 j .. 16 j + 15 (lane n -> column 16 j + n), so that the 256-frame tiles stay full
  // across row ends.  The walk is the same in every iteration, so each lane keeps, per tile, the
  // LDS offset of its operand and the offset of its 4 output frames from the iteration's first
  // row.  Columns past the R rows and frames past the end of a row get an offset that the output
  // resource rejects (a raw buffer store beyond num_records is dropped), as do rows past the
  // wave's last: no lane masking, and every iteration issues exactly g.tiles stores.
  int lds_off[kMaxTiles];
  uint32_t out_off[kMaxTiles];
#pragma unroll
  for (int j = 0; j < kMaxTiles; ++j) {
    const int col = 16 * j + n;
    const int rr = col / g.G, grp = col - rr * g.G;
    const int t = 16 * grp + 4 * gi;
    lds_off[j] = (min(rr, R - 1) * g.NCH + grp + gi) << 4;
    out_off[j] = (rr < R && t < p.Tout) ? (uint32_t)rr * (uint32_t)p.ybs + (uint32_t)t : 0xfffffff0u;
  }
  const int tiles = g.tiles;
  int8_t* const yc = p.y + (int64_t)c * p.Tout;

  auto iteration = [&](int it, int buf, auto fast_tag) {
    constexpr bool FAST = decltype(fast_tag)::value;
    const int row = s_begin + it * R;
    const unsigned char* const rows_lds = my + buf * R * rowbytes;
    wait_vm_dyn(2 * L + min(it, 2) * tiles);       // the rows of this iteration are in LDS
    asm volatile("" ::: "memory");
    if (g.dbg & 1) { issue(row + 3 * R, buf); return; }

    // ---- tiles, two per step so that the LDS reads, matrix products and rescales of independent
    // tiles overlap (an odd last tile drags along a partner whose stores are all rejected)
    const int Rv = min(R, s_end - row);
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
        yc + (int64_t)row * p.ybs, 0, (int)((uint32_t)(Rv - 1) * (uint32_t)p.ybs + (uint32_t)p.Tout), 0x00027000);
#pragma unroll
    for (int j = 0; j < kMaxTiles; j += 2) {
      if (j < tiles) {
        v4i acc[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const unsigned char* bp = rows_lds + lds_off[j + e];
          acc[e] = (v4i){bias, bias, bias, bias};
#pragma unroll
          for (int kc = 0; kc < KC; ++kc) {
            const v4i xb = *reinterpret_cast<const v4i*>(bp + kc * 64);
            acc[e] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[kc], xb, acc[e], 0, 0, 0);
          }
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int32_t a4[4] = {acc[e][0], acc[e][1], acc[e][2], acc[e][3]};
          const uint32_t pk = requant_pack4<FAST, false>(a4, mc, sh, rnd, 0u, lo, hi127);
          if (e == 0 || j + 1 < tiles)
            __builtin_amdgcn_raw_buffer_store_b32(pk, yrs, out_off[j + e], 0, 0);
        }
      }
    }
    asm volatile("" ::: "memory");                 // every LDS read of this buffer has been consumed
    issue(row + 3 * R, buf);
  };

  for (int it0 = 0; it0 < n_it; it0 += 3) {
#pragma unroll
    for (int h = 0; h < 3; ++h) {
      if (it0 + h >= n_it) break;
      if (fast) iteration(it0 + h, h, std::true_type{});
      else iteration(it0 + h, h, std::false_type{});
    }
  }
  wait_vm<0>();   // the look-ahead requests past the last iteration are still in flight
}

struct Plan { int KC, R, NI, S; };

bool plan(const ConvParams& p, DwpGeom& g, Plan& pl) {
  if (!p.depthwise || p.stride != 1 || p.Tout < 1 || p.res) return false;
  if (p.Tin % 16 != 0 || p.xbs % 16 != 0 || (uintptr_t)p.x % 16 != 0) return false;
  if (p.Tout % 4 != 0 || p.ybs % 4 != 0 || (uintptr_t)p.y % 4 != 0) return false;
  if (p.ybs >= 0x20000000LL) return false;               // row offsets within an iteration are 32-bit
  g.delta = ((-p.pl) % 16 + 16) % 16;
  g.PH = (p.pl + g.delta) / 16;
  const int64_t need = 16 + g.delta + (int64_t)p.dil * (p.k - 1);
  if (need > 256) return false;
  pl.KC = (int)((need + 63) / 64);
  g.G = (p.Tout + 15) / 16;
  g.NCH = g.G + 4 * pl.KC - 1;
  pl.NI = (g.NCH + 63) / 64;
  if (pl.NI > 2) return false;                          // longer rows: dw_mfma.hip cuts them up
  g.c_per_xcd = (p.Cout + 7) / 8;
  g.dbg = 0;
  if (const char* e = getenv("QASR_DWP_DBG")) g.dbg = atoi(e);

  // Batch splits S (workgroups per channel) and rows per iteration R: aim at >= 512 workgroups
  // with at least 3 iterations per wave; R = 2 keeps the 256-frame tiles fuller across row ends.
  const int64_t rows = p.B;
  pl.R = 1;
  pl.S = 1;
  if (pl.NI == 1 && 2 * g.G <= 16 * kMaxTiles && (int64_t)p.Cout >= 512 && rows / (4 * 2) >= 3) pl.R = 2;
  while ((int64_t)p.Cout * pl.S < 512 && rows / ((int64_t)4 * pl.R * (pl.S * 2)) >= 3) pl.S *= 2;
  if (const char* e = getenv("QASR_DWP")) {              // tuning override: "R,S"
    int r = 0, s = 0;
    if (sscanf(e, "%d,%d", &r, &s) == 2 && (r == 1 || (r == 2 && pl.NI == 1 && 2 * g.G <= 16 * kMaxTiles)) &&
        s >= 1 && s <= 64) {
      pl.R = r; pl.S = s;
    }
  }
  if (pl.R * g.G > 16 * kMaxTiles) return false;
  g.tiles = (pl.R * g.G + 15) / 16;
  if (2 * pl.R * pl.NI + 2 * g.tiles > 32) return false;   // the hand-counted waits go up to 32
  // rows per wave: the batch split over S workgroups x 4 waves, rounded up to a multiple of R
  int64_t spw = (rows + (int64_t)4 * pl.S - 1) / ((int64_t)4 * pl.S);
  spw = (spw + pl.R - 1) / pl.R * pl.R;
  g.spw = (int)spw;
  if (spw < 3 * pl.R) return false;                     // too little work per wave to pipeline
  if ((rows + 4 * spw - 1) / (4 * spw) > 65535) return false;
  return true;
}

template <int KC, int R, int NI>
hipError_t launch_t(const ConvParams& p, const DwpGeom& g, hipStream_t st) {
  const unsigned gy = (unsigned)((p.B + 4 * g.spw - 1) / (4 * g.spw));
  const dim3 grid(8 * g.c_per_xcd, gy);
  const size_t shmem = (size_t)4 * 3 * R * g.NCH * 16;
  return launch_kernel(dw_pipe_kernel<KC, R, NI>, grid, dim3(256), shmem, st, p, g);
}

template <int KC>
hipError_t launch_kc(const ConvParams& p, const DwpGeom& g, const Plan& pl, hipStream_t st) {
  if (pl.R == 2) return launch_t<KC, 2, 1>(p, g, st);
  if (pl.NI == 2) return launch_t<KC, 1, 2>(p, g, st);
  return launch_t<KC, 1, 1>(p, g, st);
}

}  // namespace

bool dw_pipe_supported(const ConvParams& p) {
  DwpGeom g;
  Plan pl;
  return plan(p, g, pl);
}

hipError_t launch_dw_pipe(const ConvParams& p, hipStream_t st) {
  DwpGeom g;
  Plan pl;
  if (!plan(p, g, pl)) return hipErrorInvalidValue;
  switch (pl.KC) {
    case 1: return launch_kc<1>(p, g, pl, st);
    case 2: return launch_kc<2>(p, g, pl, st);
    case 3: return launch_kc<3>(p, g, pl, st);
    default: return launch_kc<4>(p, g, pl, st);
  }
}

}  // namespace qasr
