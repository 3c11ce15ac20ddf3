// Pointwise (k = 1) int8 convolution  Y[co, t] = sum_ci W[co, ci] * X[ci, t]  on the gfx950 int8
// matrix cores, activation tile stationary in LDS, with the fused epilogue (bias, dyadic rescale,
// residual, clamp).
//
// Work decomposition.  The frames of all batch items are cut into groups of 16 (rows are a
// multiple of 16 frames long); a workgroup of 8 waves owns MT consecutive groups of that flat
// group list and ALL input channels of them: the [Cin][16*MT] activation tile is brought into
// LDS once, by direct global->LDS loads, and every output channel is computed from it.  HBM
// therefore sees each activation byte once.  Wave w of the workgroup owns output channels
// 16*NT*(8*pass + w) .. +16*NT of each pass over the output channels; its weights come straight
// from L2 in matrix-core operand order (1 KiB contiguous per wave-wide load, two chunks ahead).
//
// LDS layout.  Row = input channel, 128 bytes = 8 units of 16 frames.  A direct load writes
// 64 lanes x 16 bytes contiguously (8 rows), so rows cannot be padded; instead unit u of row r is
// stored in slot u ^ (r & 7).  The matrix-core operand is fetched with the LDS transpose read
// (ds_read_b64_tr_b8): within 16 lanes, lane i receives byte (i & 7) of the 8-byte row addressed
// by lane 2j + (i >> 3) as its byte j.  Lane l of a 16-lane group addresses channel row (l >> 1),
// frames 8 (l & 1)..+8, so lane m ends up with 8 consecutive channels of frame m: the A operand
// (rows = frames, K = channels) of v_mfma_i32_16x16x64_i8.  The 8 rows a 16-lane group touches
// have distinct (r & 7) and therefore distinct slots: no bank conflicts.  Lane group gi takes
// channels 8 gi..+8 and 32 + 8 gi..+8 of a 64-channel chunk, the order the packed weights use.
//
// Output path.  An accumulator lane holds 4 consecutive frames of one channel; storing those
// directly would touch 16 rows with 16 bytes each per instruction.  Each wave therefore owns a
// [16*NT channels][128 bytes] staging area in LDS (same slot swizzle): the residual tile is
// brought there by direct loads before the multiply loop starts, the epilogue adds it and puts the
// packed int8 results back in place, and the rows leave as 16-byte stores, 8 lanes per row.
#include "kernels.hpp"
#include "tuning.hpp"
#include "vmem.hpp"

#include <cstdlib>
#include <type_traits>

namespace qasr {


namespace {

struct PwtGeom {
  int G;        // 16-frame groups in total: B * Tin / 16
  int gpr;      // groups per row: Tin / 16
  int kch;      // Cin / 64
  int passes;   // ceil(Cout / (128 * NT))
  int co16n;    // ceil(Cout / 16)
  int tiles, tiles_per_xcd;
};

__device__ __forceinline__ v2i lds_read_tr8(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr8_b64_v2i32(
      (v2i __attribute__((address_space(3)))*)(const_cast<unsigned char*>(p)));
}

// Order of the vector-memory requests of a wave and the waits that follow from it (requests
// complete in order, so "at most N outstanding" means everything but the N youngest is done):
//
//   R        residual tile of pass 0 -> staging (direct)            oldest
//   C        bias, m, s of pass 0
//   W(0)     weights of chunk 0                      (NT requests)
//   X(0)     this wave's 8 rows of activation chunk 0 (direct, 1 request)
//   W(1)
//   X(1) .. X(kch-1)
//   then, after chunk q has been multiplied:  W(q+2)  (the weight stream runs on across passes)
//
//   chunk 0 needs C, W(0), X(0):  NT + kch - 1 younger requests may stay outstanding
//   chunk 1 needs W(1), X(1):     NT + kch - 2
//   chunk q >= 2 needs W(q):      NT          (W(q) is younger than every X: all of X has landed)
//
// A workgroup barrier after each of the first three waits publishes the other waves' rows.  So
// the multiplication starts as soon as the first 64 channels are there and the rest of the tile
// streams in behind it.  Later passes (Cout > 128 NT) start from a full wait.
template <int MT, int NT>
__global__ __launch_bounds__(512) void pw_tile_kernel(ConvParams p, PwtGeom g) {
  extern __shared__ __align__(128) unsigned char xs[];  // [Cin][128] slots swizzled, then staging

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, gi = lane >> 4;
  // Workgroup -> tile: the hardware deals consecutive workgroups round-robin to the 8 XCDs (each
  // with its own L2).  Neighbouring tiles share the cache lines at their common edge (a tile row is
  // 16*MT bytes at an arbitrary 16-byte offset), so each XCD gets one contiguous range of tiles:
  // the shared lines are then fetched once and written back whole.
  const int tile = (int)(blockIdx.x & 7) * g.tiles_per_xcd + (int)(blockIdx.x >> 3);
  if ((blockIdx.x >> 3) >= (unsigned)g.tiles_per_xcd || tile >= g.tiles) return;   // whole workgroup
  const int g0 = tile * MT;
  const int kch = g.kch;

  // lane -> (row lane/8 of a block of 8 rows, slot lane%8); the unit in that slot, slot ^ (row & 7),
  // is the same for every block of 8 rows, so one lane -> unit map serves the activation loads,
  // the residual loads and the output stores.
  const int u_l = (lane & 7) ^ (lane >> 3);
  const int gq_l = g0 + u_l;
  const bool u_ok = u_l < MT && gq_l < g.G;
  const int b_l = gq_l / g.gpr, t16_l = gq_l - b_l * g.gpr;
  const int64_t yoff_l = (int64_t)b_l * p.ybs + 16 * t16_l;       // of this lane's unit
  unsigned char* const stage = xs + (size_t)p.Cin * 128 + wave * (16 * NT * 128);
  int32_t* const stash = reinterpret_cast<int32_t*>(xs + (size_t)p.Cin * 128 + 8 * (16 * NT * 128)) + wave * (2 * NT * 64);

  auto load_residual = [&](int co_w) {
    if (p.res && u_ok) {
#pragma unroll
      for (int it = 0; it < 2 * NT; ++it) {
        const int co = co_w + 8 * it + (lane >> 3);
        if (co < p.Cout) direct_load16(p.res + yoff_l + (int64_t)co * p.Tout, stage + it * 1024);
      }
    }
  };
  int32_t bv[NT], mc[NT], sc[NT];
  auto load_consts = [&](int co_w) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int co = min(co_w + 16 * nt + n, p.Cout - 1);
      bv[nt] = p.bias ? gload4(p.bias + co) : 0;
      mc[nt] = gload4(p.m + co);
      sc[nt] = gload4(p.s + co);
    }
  };
  // weight stream: chunk q of the flat (pass, chunk) sequence, clamped at its end
  const int Q = g.passes * kch;
  const v4i wrsrc = make_rsrc(p.w, (uint32_t)g.co16n * (uint32_t)kch * 1024u);
  const uint32_t wlane = (uint32_t)lane * 16;
  auto load_w = [&](int q, v4i (&dst)[NT]) {
    q = min(q, Q - 1);
    const int ps = q / kch, kc = q - ps * kch;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int co16 = min((ps * 8 + wave) * NT + nt, g.co16n - 1);
      dst[nt] = bload16(wrsrc, wlane, (uint32_t)(co16 * kch + kc) * 1024u);
    }
  };

  v4i wb[2][NT];
  load_residual(wave * 16 * NT);
  load_consts(wave * 16 * NT);
  {
    const int r = 8 * wave + (lane >> 3);
    const int8_t* src = p.x + (int64_t)b_l * p.xbs + (int64_t)r * p.Tin + 16 * t16_l;
    const int64_t step = (int64_t)64 * p.Tin;
    unsigned char* dst = xs + 8 * wave * 128;
    load_w(0, wb[0]);
    if (u_ok) direct_load16(src, dst);
    load_w(1, wb[1]);
    for (int kc = 1; kc < kch; ++kc)
      if (u_ok) direct_load16(src + kc * step, dst + kc * 8192);
  }

  // per-lane constants of the transpose reads and of the staging writes
  const int l16 = lane & 15, j = l16 >> 1;
  // Slot of unit mt in row r is mt ^ (r & 7): with the row's own (r & 7) << 4 folded into the
  // lane's base offset, the address of unit mt is base ^ (mt << 4)  (LDS tile is 128-byte aligned).
  const uint32_t abase = (uint32_t)((8 * gi + j) * 128 + 8 * (l16 & 1)) | (uint32_t)(j << 4);
  const uint32_t sbase = (uint32_t)(n * 128 + 4 * gi) | (uint32_t)((n & 7) << 4);   // staging row 16 nt + n
  const int lo = p.relu ? 0 : -128;

  int q = 0;
  for (int ps = 0; ps < g.passes; ++ps) {
    const int co_w = (ps * 8 + wave) * 16 * NT;       // wave-uniform
    const bool active = co_w < p.Cout;                // idle waves still load and synchronise
    if (ps > 0) {
      load_residual(co_w);
      load_consts(co_w);
      wait_vm<0>();
    }
    v4i acc[MT][NT];

    for (int kc = 0; kc < kch; kc += 2) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kk = kc + h;                        // kch is even
        if (ps == 0 && kk < 2) {
          wait_vm_dyn(NT + kch - 1 - kk);
        } else if (!(ps > 0 && kk == 0)) {
          wait_vm<NT>();
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) tie(wb[h][nt]);
        if (ps == 0 && kk <= 2) __syncthreads();
        if (kk == 0) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            tie(bv[nt]); tie(mc[nt]); tie(sc[nt]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = (v4i){bv[nt], bv[nt], bv[nt], bv[nt]};
            stash[(2 * nt) * 64 + lane] = mc[nt];       // parked in LDS until the epilogue
            stash[(2 * nt + 1) * 64 + lane] = sc[nt];
          }
        }
        if (active) {
          // the activation operand of the next 16-frame group is read from LDS while the current
          // one is multiplied; the scheduling fences keep that order
          const unsigned char* ab = xs + kk * 8192;
          v2i a0 = lds_read_tr8(ab + abase);
          v2i a1 = lds_read_tr8(ab + abase + 4096);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const v4i a = {a0.x, a0.y, a1.x, a1.y};
            if (mt + 1 < MT) {
              a0 = lds_read_tr8(ab + (abase ^ ((mt + 1) << 4)));
              a1 = lds_read_tr8(ab + (abase ^ ((mt + 1) << 4)) + 4096);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, wb[h][nt], acc[mt][nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        load_w(q + 2, wb[h]);
        ++q;
      }
    }

    // ---- epilogue: lane (n, gi) holds frames 16 mt + 4 gi + (0..3) of channel co_w + 16 nt + n
    if (!active) continue;
    bool fast = true;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      mc[nt] = stash[(2 * nt) * 64 + lane];
      sc[nt] = stash[(2 * nt + 1) * 64 + lane];
      fast = fast && sc[nt] >= 33;
    }
    const bool all_fast = __all(fast);                  // wave-uniform: one code path
    // Two variants only (all s >= 33, or the 64-bit form); the residual bytes are always added
    // (zeros when there is no residual): more variants would share sub-expressions, which the
    // compiler then hoists above the selecting branch for all accumulators at once.
    const bool has_res = p.res != nullptr;
    auto epilogue = [&](auto fast_tag) {
      constexpr bool FAST = decltype(fast_tag)::value;
      const int32_t hi127 = 127;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int sh = FAST ? sc[nt] - 32 : sc[nt], rnd = FAST ? 1 << (sc[nt] - 33) : 0;
        uint32_t rw[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) rw[mt] = 0u;
        if (has_res) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            rw[mt] = *reinterpret_cast<const uint32_t*>(stage + nt * 2048 + (sbase ^ (mt << 4)));
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int32_t a4[4] = {acc[mt][nt][0], acc[mt][nt][1], acc[mt][nt][2], acc[mt][nt][3]};
          *reinterpret_cast<uint32_t*>(stage + nt * 2048 + (sbase ^ (mt << 4))) =
              requant_pack4<FAST, true>(a4, mc[nt], sh, rnd, rw[mt], lo, hi127);
          if (mt & 1) __builtin_amdgcn_sched_barrier(0);   // bounds the live temporaries
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if (all_fast) epilogue(std::true_type{}); else epilogue(std::false_type{});
    // rows out: lane -> (row 8 it + lane/8, slot lane%8) = unit u_l of channel co_w + row
#pragma unroll
    for (int it = 0; it < 2 * NT; ++it) {
      const v4i o = *reinterpret_cast<const v4i*>(stage + it * 1024 + lane * 16);
      const int co = co_w + 8 * it + (lane >> 3);
      if (u_ok && co < p.Cout) *reinterpret_cast<v4i*>(p.y + yoff_l + (int64_t)co * p.Tout) = o;
    }
  }
  // The clamped tail of the weight stream is still in flight: let it land, with the ring's
  // registers still the ring's (an unread asm output is dead to the compiler, which would reuse
  // the registers while the data is on its way).
  wait_vm<0>();
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) tie(wb[h][nt]);
}

struct Choice { int MT, NT; };

// activation tile + per-wave staging + per-wave park space for m and s
size_t lds_bytes(const ConvParams& p, int NT) { return (size_t)p.Cin * 128 + (size_t)8 * 16 * NT * 128 + (size_t)8 * 2 * NT * 64 * 4; }

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
  if (p.Tin % 16) return false;
  const int64_t G = (int64_t)p.B * (p.Tin / 16);
  if (G > 0x3fffffff) return false;
  c.NT = p.Cout > 256 ? 4 : (p.Cout > 128 ? 2 : 1);
  while (c.NT > 1 && lds_bytes(p, c.NT) > 160 * 1024) c.NT >>= 1;   // narrower passes: smaller staging
  if (lds_bytes(p, c.NT) > 160 * 1024) return false;
  // groups per tile: least makespan over the CUs (one workgroup per CU at a time), with a
  // per-tile overhead worth about one group
  double best = 1e300;
  for (int MT = 4; MT <= 8; ++MT) {
    const int64_t tiles = (G + MT - 1) / MT;
    const double cost = (double)((tiles + cus - 1) / cus) * (MT + 1.0);
    if (cost < best - 1e-9) { best = cost; c.MT = MT; }
  }
  {                                                     // tuning override
    const int mt = tuning().pwt_mt;
    if (mt >= 4 && mt <= 8) c.MT = mt;
  }
  return true;
}

template <int MT, int NT>
hipError_t launch_t(const ConvParams& p, hipStream_t st) {
  PwtGeom g;
  g.gpr = p.Tin / 16;
  g.G = p.B * g.gpr;
  g.kch = p.Cin / 64;
  g.passes = (p.Cout + 128 * NT - 1) / (128 * NT);
  g.co16n = (p.Cout + 15) / 16;
  const size_t shmem = lds_bytes(p, NT);
  static std::atomic<uint64_t> lds_raised{0};   // per instantiation, a bit per device
  if (const hipError_t e = ensure_max_dynamic_lds((const void*)pw_tile_kernel<MT, NT>, lds_raised); e != hipSuccess)
    return e;
  g.tiles = (g.G + MT - 1) / MT;
  g.tiles_per_xcd = (g.tiles + 7) / 8;
  return launch_kernel(pw_tile_kernel<MT, NT>, dim3((unsigned)(8 * g.tiles_per_xcd)), dim3(512), shmem, st, p, g);
}

}  // namespace

bool pw_tile_supported(const ConvParams& p) {
  if (p.depthwise || p.k != 1 || p.stride != 1 || p.pl != 0 || p.Tout != p.Tin) return false;
  if (!p.w_packed || p.Cin % 128 != 0 || p.Cin > 1024 || p.Tin % 16 != 0) return false;
  if (p.xbs % 16 != 0 || p.ybs % 16 != 0) return false;
  if ((uintptr_t)p.x % 16 || (uintptr_t)p.y % 16 || (uintptr_t)p.w % 16 || (p.res && (uintptr_t)p.res % 16))
    return false;
  Choice c;
  return pick(p, c, 256);
}

hipError_t launch_pw_tile(const ConvParams& p, hipStream_t st) {
  Choice c;
  if (!pw_tile_supported(p) || !pick(p, c, num_cus())) return hipErrorInvalidValue;
#define QASR_CASE(M, N) if (c.MT == M && c.NT == N) return launch_t<M, N>(p, st);
  QASR_CASE(4, 1) QASR_CASE(4, 2) QASR_CASE(4, 4)
  QASR_CASE(5, 1) QASR_CASE(5, 2) QASR_CASE(5, 4)
  QASR_CASE(6, 1) QASR_CASE(6, 2) QASR_CASE(6, 4)
  QASR_CASE(7, 1) QASR_CASE(7, 2) QASR_CASE(7, 4)
  QASR_CASE(8, 1) QASR_CASE(8, 2) QASR_CASE(8, 4)
#undef QASR_CASE
  return hipErrorInvalidValue;
}

}  // namespace qasr
