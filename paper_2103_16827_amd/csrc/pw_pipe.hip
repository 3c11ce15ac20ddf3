// Pointwise (k = 1) int8 convolution  Y[co, t] = sum_ci W[co, ci] * X[ci, t]  on the gfx950 int8
// matrix cores, activation tile stationary in LDS, output channels in software-pipelined passes,
// with the fused epilogue (bias, dyadic rescale, residual, clamp).
//
// Tile, LDS layout, transpose reads, weight stream and staging are those of pw_tile.hip: a
// workgroup of 8 waves owns MT consecutive 16-frame groups and all input channels of them; wave w
// computes output channels 32 * (8 * pass + w) .. + 32 in pass `pass`.  What is different is the
// order of work inside a wave.  In pw_tile a wave multiplies, then rescales and stores, and since
// the two waves that share a SIMD do the same, the matrix pipeline idles during every epilogue.
// Here the epilogue of pass p - 1 (accumulator set (p - 1) mod 2) is issued in between the matrix
// products of pass p: a wave issues in order, so vector instructions placed between two products
// execute while the first one occupies the matrix pipeline.  Every chunk step of the multiply
// loop (64 input channels: MT transpose-read pairs, 2 MT products) carries its share of the 2 MT
// epilogue blocks of the pass before, as steps of three mutually independent vector instructions;
// scheduling fences pin the pattern   product, step | product, step | ...
// The rows of pass p - 1 leave at the end of pass p's loop and drain under pass p + 1.  Only the
// last pass's epilogue is exposed.  A pass whose s values are not all >= 33 (64-bit rescale), or a
// layer without relu, is not pipelined: its epilogue follows its own loop, as in pw_tile.
//
// Vector-memory completion is tracked by hand (vmem.hpp): the wave counts the requests it issues
// (`seq`) and remembers the count after each request it will wait for, so "everything up to that
// request has completed" is  vmcnt(seq - mark).  Nothing that is in flight lives in a compiler
// variable across the pass loop except the two weight buffers, whose every use follows a tie().
#include "kernels.hpp"
#include "vmem.hpp"
#include "tuning.hpp"
#include "pw_pipe_body.hpp"

#include <cstdlib>
#include <type_traits>

namespace qasr {

namespace {

using namespace pwp;

// ACT: a unary activation's table is applied after the clamp (an instantiation of its own: the
// plain layers keep their code as it is)
template <int MT, int KCH, bool ACT>
__global__ __launch_bounds__(512) void pw_pipe_kernel(ConvParams p, PwpGeom g) {
  extern __shared__ __align__(128) unsigned char xs[];
  pw_pipe_tile<MT, KCH, ACT, false>(p, g, blockIdx.x, xs, (int)threadIdx.x);
}

// The lean form: one pass per workgroup, two workgroups per compute unit (four waves per SIMD:
// at most 128 registers each).
template <int MT, int KCH>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(4, 4)))
void pw_lean_kernel(ConvParams p, PwpGeom g) {
  extern __shared__ __align__(128) unsigned char xs[];
  pw_pipe_tile<MT, KCH, false, false, 2, true>(p, g, blockIdx.x, xs, (int)threadIdx.x);
}

struct Choice { int MT, KCH, splits; bool lean; };

size_t lds_bytes(int KCH) { return KCH == 4 ? lds_bytes_c<4>() : lds_bytes_c<8>(); }   // (8 chunks at most are resident)

int num_cus() {
  static int n = 0;
  if (!n) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
    else
      n = 256;
  }
  return n;
}

// Shape-only part of the choice (no device query: usable without a GPU).
bool pick(const ConvParams& p, Choice& c, int cus) {
  if (tuning().no_pw_pipe) return false;                  // tuning: fall through to the other kernels
  if (p.depthwise || p.k != 1 || p.stride != 1 || p.pl != 0 || p.Tout != p.Tin) return false;
  if (!p.w_packed || p.Tin % 16 != 0) return false;
  if (p.Cin != 256 && p.Cin != 512 && p.Cin != 1024 && p.Cin != 2048) return false;   // instantiated widths
  if (p.Cin > 512 && p.Cout % (8 * ROWS) != 0) return false;   // streamed input: one pass per workgroup, whole passes only
  if (p.Cout < 8 * ROWS || p.Cout > MAXP * 8 * ROWS) return false;   // every wave has channels in pass 0
  if (p.xbs % 16 != 0 || p.ybs % 16 != 0) return false;
  if ((uintptr_t)p.x % 16 || (uintptr_t)p.y % 16 || (uintptr_t)p.w % 16 || (p.res && (uintptr_t)p.res % 16))
    return false;
  if ((int64_t)p.B * p.ybs >= 0x7ffffff0LL) return false;          // 32-bit output offsets
  const int64_t G = (int64_t)p.B * (p.Tin / 16);
  if (G > 0x3fffffff) return false;
  c.KCH = p.Cin / 64;
  // groups per tile: least makespan over the CUs (one workgroup per CU at a time), with a
  // per-tile overhead worth about one group
  // and, when the tiles do not fill the CUs, workgroups per tile (each takes passes / splits
  // passes of 256 channels and loads the tile again).  Times in microseconds fitted to single-layer
  // measurements at 512 input channels (B=16, T=400; 2048, 1024 and 512 output channels): a
  // workgroup takes about 6.5 + passes * (0.5 MT + 0.7); the per-pass part halves at 256 channels.
  const int passes = (p.Cout + 8 * ROWS - 1) / (8 * ROWS);
  const double kscale = c.KCH / 8.0;
  double best = 1e300;
  c.MT = 7;
  c.splits = 1;
  for (int splits = 1; splits <= passes; splits *= 2) {
    if (passes % splits != 0 || (splits > 1 && p.Cout % (8 * ROWS) != 0)) continue;
    if (c.KCH > 8 && splits != passes) continue;            // streamed input: exactly one pass per workgroup
    for (int MT = 4; MT <= kMaxMT; ++MT) {
      const int64_t wgs = (G + MT - 1) / MT * splits;
      const double cost = (double)((wgs + cus - 1) / cus) * (6.5 + (passes / splits) * kscale * (0.5 * MT + 0.7));
      if (cost < best - 1e-9) { best = cost; c.MT = MT; c.splits = splits; }
    }
  }
  if (passes & (passes - 1)) {                              // (splits run over powers of two)
    if (c.KCH > 8) return false;
  }
  // The lean form (every pass a workgroup of its own, two workgroups per unit) for layers without a
  // fused activation whose tile stays resident, when all its workgroups are resident at once: 7 groups per tile.  Single
  // layers at B=32, T=800 against the form above: 256->256 13.0 against 14.0 us, 256->512 14.9
  // against 17.5, 512->512 13.8 against 15.4, 512->1024 (two rounds) no difference; smaller tiles
  // are slower (more workgroups than resident slots, or the weights streamed more often).  Launches
  // that leave most units empty keep the pipelined form (batch 1: 0.313 against 0.330 ms for the
  // QuartzNet-5x5 shape).
  const int64_t lean_wgs = ((G + kMaxMT - 1) / kMaxMT) * passes;
  c.lean = !tuning().no_pw_lean && !(p.res && tuning().pw_lean_no_res) && !p.act_lut && c.KCH <= 8 &&
           p.Cout % (8 * ROWS) == 0 &&
           (tuning().pw_lean_force || (2 * lean_wgs > cus && lean_wgs <= 2 * (int64_t)cus));
  if (c.lean) { c.splits = passes; c.MT = kMaxMT; }
  {                                                       // tuning overrides
    const int mt = tuning().pwp_mt, sp = tuning().pwp_split;
    if (mt >= 4 && mt <= kMaxMT) c.MT = mt;
    if (!c.lean && sp >= 1 && passes % sp == 0 && (sp == 1 || p.Cout % (8 * ROWS) == 0) && c.KCH <= 8) c.splits = sp;
  }
  return lds_bytes(c.KCH) <= 160 * 1024;
}

template <int MT, int KCH, bool ACT>
hipError_t launch_a(const ConvParams& p, int splits, hipStream_t st) {
  PwpGeom g;
  g.gpr = p.Tin / 16;
  g.G = p.B * g.gpr;
  g.passes = (p.Cout + 8 * ROWS - 1) / (8 * ROWS);
  g.co16n = (p.Cout + 15) / 16;
  g.tiles = (g.G + MT - 1) / MT;
  g.tiles_per_xcd = (g.tiles + 7) / 8;
  g.splits = splits;
  g.pps = g.passes / splits;
  g.nopipe = tuning().pwp_nopipe ? 1 : 0;
  static std::atomic<uint64_t> lds_raised{0};   // per instantiation, a bit per device
  if (const hipError_t e = ensure_max_dynamic_lds((const void*)pw_pipe_kernel<MT, KCH, ACT>, lds_raised); e != hipSuccess)
    return e;
  return launch_kernel(pw_pipe_kernel<MT, KCH, ACT>, dim3((unsigned)(8 * g.tiles_per_xcd * g.splits)), dim3(512),
                       (size_t)lds_bytes_c<KCH>(), st, p, g);
}

template <int MT, int KCH>
hipError_t launch_lean(const ConvParams& p, hipStream_t st) {
  PwpGeom g;
  g.gpr = p.Tin / 16;
  g.G = p.B * g.gpr;
  g.passes = p.Cout / (8 * ROWS);
  g.co16n = (p.Cout + 15) / 16;
  g.tiles = (g.G + MT - 1) / MT;
  g.tiles_per_xcd = (g.tiles + 7) / 8;
  g.splits = g.passes;
  g.pps = 1;
  g.nopipe = 1;
  static std::atomic<uint64_t> lds_raised{0};
  if (const hipError_t e = ensure_max_dynamic_lds((const void*)pw_lean_kernel<MT, KCH>, lds_raised, lds_bytes_lean_c<KCH>());
      e != hipSuccess)
    return e;
  return launch_kernel(pw_lean_kernel<MT, KCH>, dim3((unsigned)(8 * g.tiles_per_xcd * g.splits)), dim3(512),
                       (size_t)lds_bytes_lean_c<KCH>(), st, p, g);
}

template <int MT, int KCH>
hipError_t launch_t(const ConvParams& p, int splits, hipStream_t st) {
  return p.act_lut ? launch_a<MT, KCH, true>(p, splits, st) : launch_a<MT, KCH, false>(p, splits, st);
}

}  // namespace

bool pw_pipe_supported(const ConvParams& p) {
  Choice c;
  return pick(p, c, 256);
}

hipError_t launch_pw_pipe(const ConvParams& p, hipStream_t st) {
  Choice c;
  if (!pick(p, c, num_cus())) return hipErrorInvalidValue;
#define QASR_CASE(M, K) if (c.lean && c.MT == M && c.KCH == K) return launch_lean<M, K>(p, st);
  QASR_CASE(4, 4) QASR_CASE(5, 4) QASR_CASE(6, 4) QASR_CASE(7, 4)
  QASR_CASE(4, 8) QASR_CASE(5, 8) QASR_CASE(6, 8) QASR_CASE(7, 8)
#undef QASR_CASE
#define QASR_CASE(M, K) if (c.MT == M && c.KCH == K) return launch_t<M, K>(p, c.splits, st);
  QASR_CASE(4, 4) QASR_CASE(5, 4) QASR_CASE(6, 4) QASR_CASE(7, 4)
  QASR_CASE(4, 8) QASR_CASE(5, 8) QASR_CASE(6, 8) QASR_CASE(7, 8)
  QASR_CASE(4, 16) QASR_CASE(5, 16) QASR_CASE(6, 16) QASR_CASE(7, 16)
  QASR_CASE(4, 32) QASR_CASE(5, 32) QASR_CASE(6, 32) QASR_CASE(7, 32)
#undef QASR_CASE
  return hipErrorInvalidValue;
}

}  // namespace qasr
