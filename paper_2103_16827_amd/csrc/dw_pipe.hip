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
// outstanding:  loads(i+1), loads(i+2) [L each] + stores(i-2), stores(i-1) [one per 256-frame tile
// of the iteration's whole pairs of tiles].
// Needs 16-byte aligned rows that are a multiple of 16 frames and at most ~1000 frames long,
// 4-byte aligned outputs and no residual operand; everything else is served by dw_mfma.hip.
#include "kernels.hpp"
#include "vmem.hpp"
#include "tuning.hpp"

#include <cstdio>
#include <cstdlib>
#include <type_traits>

namespace qasr {

namespace {

// cache policy of the output stores (sc0 sc1): written through towards memory as they are issued,
// so that little is left to write back when the kernel ends
constexpr int kStoreThrough = 17;
constexpr int kMaxTiles = 8; // 256-frame tiles per iteration: R * groups per strip <= 128

struct DwpGeom {
  int delta;      // (-pad_left) mod 16
  int PH;         // (pad_left + delta) / 16: left halo in 16-byte chunks
  int NCH;        // 16-byte chunks per strip buffer: groups + 4*KC - 1
  int G;          // 16-frame groups per row
  int tiles;      // 256-frame tiles per iteration: ceil(R * G / 16) <= kMaxTiles
  int spw;        // rows per wave (a multiple of R)
  int c_per_xcd;  // channels per XCD: ceil(C / 8)
};

// ACT: a unary activation's table is applied after the clamp (its own instantiation: the plain
// layers keep their code as it is)
template <int KC, int R, int NI, bool ACT>
__global__ __launch_bounds__(256) void dw_pipe_kernel(ConvParams p, DwpGeom g) {
  extern __shared__ __align__(16) unsigned char strips_lds[];      // [4 waves][3 buffers][R][NCH][16]
  __shared__ __align__(16) unsigned char a_lds[KC * 1024];         // A operand, register layout
  __shared__ __align__(16) unsigned char lut_lds[ACT ? 4 * 256 : 16];   // a fused activation's table, one copy per wave

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

  // Requests of one iteration (always L of them, see below): rows `row` .. `row + R - 1` into buffer `buf`.
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
  // A request in which no lane takes part is not issued at all (the compiler branches around it),
  // so only the 64-chunk slices of a row that hold at least one chunk of data count.
  int L = 0;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
    if (__builtin_amdgcn_readfirstlane((int)(__ballot(lane_in[ni]) != 0))) L += R;
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
  // The channel's weights are requested before the rows: requests complete in order, so the
  // Toeplitz operand can be built while the rows are still on their way.
  // (So are the channel's constants: loads the compiler knew of would make it wait for every
  // request of the wave, rows included, at their first use.)
  int32_t bias = 0, mc = gload4(p.m + c), sc = gload4(p.s + c);
  if (p.bias) bias = gload4(p.bias + c);
  int32_t wj = 0;
  if (tid < p.k) wj = gload_i8(p.w + (int64_t)c * p.k + tid);
  // a unary activation applied after the clamp: its 256-entry table (int8 output per int8 code),
  // 64 lanes x 4 bytes straight into this wave's copy; one more request ahead of the rows
  constexpr bool has_act = ACT;
  unsigned char* const lutw = lut_lds + (ACT ? wave * 256 : 0);
  if (has_act) direct_load4(p.act_lut + 4 * lane, lutw);
  int n_rows = 0;                               // row requests of this wave so far
  // Only the first iteration's rows are requested now, the other two after the operand is built:
  // all waves of the chip start together, and a request waits behind everything that entered
  // the memory system before it, so what is needed first has to be asked for first chip-wide.
  if (s_begin < s_end) {          // (a wave without rows issues nothing and skips the loop below)
    n_rows = L;
    issue(s_begin, 0);
  }

  // The 16-frame groups of an iteration's R rows form one flat list of columns; tile j takes
  // columns 16 j .. 16 j + 15 (lane n -> column 16 j + n), so that the 256-frame tiles stay full
  // across row ends.  The walk is the same in every iteration, so each lane keeps, per tile, the
  // LDS offset of its operand and the offset of its 4 output frames from the iteration's first
  // row.  Columns past the R rows and frames past the end of a row get an offset that the output
  // resource rejects (a raw buffer store beyond num_records is dropped), as do rows past the
  // wave's last: no lane masking.  Tiles are taken in pairs and every iteration issues exactly
  // 2 * pairs stores (an odd last tile drags along a partner whose stores are all rejected).
  int lds_off[kMaxTiles];
  uint32_t out_off[kMaxTiles];
#pragma unroll
  for (int j = 0; j < kMaxTiles; ++j) {
    int rr = 0, grp = 16 * j + n;               // column -> (row, group): at most R rows count
#pragma unroll
    for (int q = 0; q < R; ++q)
      if (grp >= g.G) { grp -= g.G; ++rr; }
    const bool in = rr < R && grp < g.G;
    if (!in) { rr = R - 1; grp = 0; }           // reads stay inside the buffer, the store is rejected
    const int t = 16 * grp + 4 * gi;
    lds_off[j] = (rr * g.NCH + grp + gi) << 4;
    out_off[j] = (in && t < p.Tout) ? (uint32_t)rr * (uint32_t)p.ybs + (uint32_t)t : 0xfffffff0u;
  }

  // ---- Toeplitz operand in the register layout of the matrix product: lane (m, gi) holds
  // A[m, 64 kc + 16 gi + (0..15)].  Weight j sits at kappa = m + delta + j * dilation for every m:
  // the thread that loaded it writes those 16 bytes into the zeroed image.
#pragma unroll
  for (int kc = 0; kc < KC; ++kc)
    reinterpret_cast<uint32_t*>(a_lds)[kc * 256 + tid] = 0u;
  __syncthreads();
  wait_vm_dyn(n_rows);                          // everything requested before the rows is here
  tie(wj); tie(bias); tie(mc); tie(sc);
  if (tid < p.k) {
    const int kap0 = g.delta + tid * p.dil;
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const int kap = kap0 + m;
      a_lds[(kap >> 6) * 1024 + (((kap >> 4) & 3) * 16 + m) * 16 + (kap & 15)] = (unsigned char)wj;
    }
  }
  __syncthreads();
  if (s_begin < s_end) {
    issue(s_begin + R, 1);
    issue(s_begin + 2 * R, 2);
  }
  v4i a[KC];
#pragma unroll
  for (int kc = 0; kc < KC; ++kc) a[kc] = *reinterpret_cast<const v4i*>(a_lds + kc * 1024 + lane * 16);

  const int lo = p.relu ? 0 : -128;
  const int32_t hi127 = 127;
  const bool fast = sc >= 33;                           // uniform: one channel per workgroup
  const int sh = fast ? sc - 32 : sc, rnd = fast ? 1 << (sc - 33) : 0;

  const int pairs = (g.tiles + 1) >> 1;
  int8_t* const yc = p.y + (int64_t)c * p.Tout;

  // One iteration, software-pipelined over its NP tile pairs: the matrix products of pair q are
  // issued, then the operands of pair q + 1 are read from LDS, then pair q - 1 is rescaled and
  // stored, so that LDS and matrix-pipeline latencies pass under the vector arithmetic.
  auto iteration = [&](int it, int buf, auto fast_tag, auto np_tag) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast_tag)::value;
    constexpr int NP = decltype(np_tag)::value;
    const int row = s_begin + it * R;
    const unsigned char* const rows_lds = my + buf * R * rowbytes;
    wait_vm_dyn(2 * L + min(it, 2) * 2 * NP);      // the rows of this iteration are in LDS
    asm volatile("" ::: "memory");

    const int Rv = min(R, s_end - row);
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
        yc + (int64_t)row * p.ybs, 0, (int)((uint32_t)(Rv - 1) * (uint32_t)p.ybs + (uint32_t)p.Tout), 0x00027000);
    const v4i bias4 = {bias, bias, bias, bias};
    v4i xb[2][2][KC];                              // [pair parity][tile of the pair][chunk]
    v4i acc[2][2];
    auto read_pair = [&](int q) __attribute__((always_inline)) {
#pragma unroll
      for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
          xb[q & 1][e][kc] = *reinterpret_cast<const v4i*>(rows_lds + lds_off[2 * q + e] + kc * 64);
    };
    auto multiply_pair = [&](int q) __attribute__((always_inline)) {
#pragma unroll
      for (int kc = 0; kc < KC; ++kc)
#pragma unroll
        for (int e = 0; e < 2; ++e)
          acc[q & 1][e] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[kc], xb[q & 1][e][kc], kc == 0 ? bias4 : acc[q & 1][e], 0, 0, 0);
    };
    auto finish_pair = [&](int q) __attribute__((always_inline)) {
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const v4i av = acc[q & 1][e];
        const int32_t a4[4] = {av[0], av[1], av[2], av[3]};
        uint32_t pk = requant_pack4<FAST, false>(a4, mc, sh, rnd, 0u, lo, hi127);
        if (has_act) {                               // table[code + 128], byte by byte
          const uint32_t cd = pk ^ 0x80808080u;
          pk = (uint32_t)lutw[cd & 0xffu] | ((uint32_t)lutw[(cd >> 8) & 0xffu] << 8) |
               ((uint32_t)lutw[(cd >> 16) & 0xffu] << 16) | ((uint32_t)lutw[cd >> 24] << 24);
        }
        __builtin_amdgcn_raw_buffer_store_b32(pk, yrs, out_off[2 * q + e], 0, kStoreThrough);
      }
    };
    read_pair(0);
#pragma unroll
    for (int q = 0; q < NP; ++q) {
      multiply_pair(q);
      if (q + 1 < NP) read_pair(q + 1);
      if (q > 0) finish_pair(q - 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    finish_pair(NP - 1);
    asm volatile("" ::: "memory");                 // every LDS read of this buffer has been consumed
    issue(row + 3 * R, buf);
  };
  auto run = [&](auto fast_tag, auto np_tag) __attribute__((always_inline)) {
    for (int it0 = 0; it0 < n_it; it0 += 3) {
#pragma unroll
      for (int h = 0; h < 3; ++h) {
        if (it0 + h >= n_it) break;
        iteration(it0 + h, h, fast_tag, np_tag);
      }
    }
  };
  auto run_np = [&](auto np_tag) __attribute__((always_inline)) {
    if (fast) run(std::true_type{}, np_tag); else run(std::false_type{}, np_tag);
  };
  switch (pairs) {
    case 1: run_np(std::integral_constant<int, 1>{}); break;
    case 2: run_np(std::integral_constant<int, 2>{}); break;
    case 3: run_np(std::integral_constant<int, 3>{}); break;
    default: run_np(std::integral_constant<int, 4>{}); break;
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

  // Batch splits S (workgroups per channel) and rows per iteration R.  Measured on the 512- and
  // 256-channel layers at batch 32: about 1024 workgroups (4 waves per SIMD) with one row per
  // iteration beat fewer, longer-running waves; two rows per iteration (fuller 256-frame tiles
  // across row ends) only pay once a wave has many iterations.
  const int64_t rows = p.B;
  pl.R = 1;
  pl.S = 1;
  while ((int64_t)p.Cout * pl.S < 1024 && rows / ((int64_t)4 * (pl.S * 2)) >= 3) pl.S *= 2;
  if (pl.NI == 1 && 2 * g.G <= 16 * kMaxTiles && rows / ((int64_t)4 * pl.S) >= 12) pl.R = 2;
  {                                                      // tuning override: "R,S"
    const int r = tuning().dwp_r, s = tuning().dwp_s;
    if ((r == 1 || (r == 2 && pl.NI == 1 && 2 * g.G <= 16 * kMaxTiles)) && s >= 1 && s <= 64) {
      pl.R = r; pl.S = s;
    }
  }
  if (pl.R * g.G > 16 * kMaxTiles) return false;
  g.tiles = (pl.R * g.G + 15) / 16;
  if (2 * pl.R * pl.NI + 4 * ((g.tiles + 1) / 2) > 32) return false;   // the hand-counted waits go up to 32
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
  if (p.act_lut) return launch_kernel(dw_pipe_kernel<KC, R, NI, true>, grid, dim3(256), shmem, st, p, g);
  return launch_kernel(dw_pipe_kernel<KC, R, NI, false>, grid, dim3(256), shmem, st, p, g);
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
