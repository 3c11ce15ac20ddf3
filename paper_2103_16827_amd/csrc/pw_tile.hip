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

#include <cstdlib>
#include <type_traits>

namespace qasr {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

namespace {

struct PwtGeom {
  int G;        // 16-frame groups in total: B * Tin / 16
  int gpr;      // groups per row: Tin / 16
  int kch;      // Cin / 64
  int passes;   // ceil(Cout / (128 * NT))
  int co16n;    // ceil(Cout / 16)
  int dbg;      // tuning: 1 skip activation loads, 2 skip multiply loop, 4 skip epilogue
};

__device__ __forceinline__ v2i lds_read_tr8(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr8_b64_v2i32(
      (v2i __attribute__((address_space(3)))*)(const_cast<unsigned char*>(p)));
}

// 64 lanes x 16 bytes from per-lane global addresses to LDS at lds_wave_base + 16 * lane
// (lds_wave_base must be wave-uniform).  Completion is counted by vmcnt.
__device__ __forceinline__ void direct_load16(const void* gptr, const unsigned char* lds_wave_base) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)lds_wave_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(gptr), "s"(m0v) : "memory");
}

template <int MT, int NT>
__global__ __launch_bounds__(512) void pw_tile_kernel(ConvParams p, PwtGeom g) {
  extern __shared__ __align__(16) unsigned char xs[];   // [Cin][128], slots swizzled

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, gi = lane >> 4;
  const int g0 = blockIdx.x * MT;

  // ---- 1. activation tile: lane -> (row 8 wave + lane/8 of each chunk, slot lane%8).  The unit
  // a lane handles, u = slot ^ (row & 7), is the same for every row block of 8, so the same
  // lane -> unit map serves the residual loads and the output stores of the staging area.
  const int u_l = (lane & 7) ^ (lane >> 3);
  const int gq_l = g0 + u_l;
  const bool u_ok = u_l < MT && gq_l < g.G;
  const int b_l = gq_l / g.gpr, t16_l = gq_l - b_l * g.gpr;
  if (u_ok && !(g.dbg & 1)) {
    const int r = 8 * wave + (lane >> 3);
    const int8_t* src = p.x + (int64_t)b_l * p.xbs + (int64_t)r * p.Tin + 16 * t16_l;
    const int64_t step = (int64_t)64 * p.Tin;
    unsigned char* dst = xs + 8 * wave * 128;
    for (int kc = 0; kc < g.kch; ++kc) {
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src + kc * step),
          (__attribute__((address_space(3))) void*)(dst + kc * 8192), 16, 0, 0);
    }
  }
  const int64_t yoff_l = (int64_t)b_l * p.ybs + 16 * t16_l;       // of this lane's unit
  unsigned char* const stage = xs + (size_t)p.Cin * 128 + wave * (16 * NT * 128);

  // ---- 2. per-lane constants of the transpose reads and of the output rows
  const int l16 = lane & 15, j = l16 >> 1;
  const unsigned char* abase = xs + (8 * gi + j) * 128 + 8 * (l16 & 1);
  int aoff[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) aoff[mt] = (mt ^ j) << 4;

  // staging address of this lane's accumulator dwords: row 16 nt + n, slot mt ^ (n & 7), + 4 gi
  int soff[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) soff[mt] = n * 128 + ((mt ^ (n & 7)) << 4) + 4 * gi;

  const int lo = p.relu ? 0 : -128;
  const int64_t wlane = (int64_t)lane * 16;

  auto w_ptr = [&](int ps, int nt) {
    const int co16 = min((ps * 8 + wave) * NT + nt, g.co16n - 1);
    return p.w + (int64_t)co16 * g.kch * 1024 + wlane;
  };

  // Residual tile of one pass -> staging area, by direct loads.  Issued through inline assembly:
  // the compiler then keeps its load counters exact for the weight prefetches of the multiply
  // loop (it cannot see these requests, which only makes its own waits stricter, never weaker);
  // the epilogue waits for them explicitly.
  auto load_residual = [&](int co_w) {
    if (p.res && u_ok) {
#pragma unroll
      for (int it = 0; it < 2 * NT; ++it) {
        const int co = co_w + 8 * it + (lane >> 3);
        if (co < p.Cout)
          direct_load16(p.res + yoff_l + (int64_t)co * p.Tout, stage + it * 1024);
      }
    }
  };
  load_residual(wave * 16 * NT);

  __builtin_amdgcn_s_waitcnt(0);   // all of this wave's direct loads have landed in LDS
  __syncthreads();

  for (int ps = 0; ps < g.passes; ++ps) {
    const int co_w = (ps * 8 + wave) * 16 * NT;       // wave-uniform
    if (co_w >= p.Cout) break;

    const int8_t* wp[NT];
    int32_t mc[NT], sc[NT];
    v4i acc[MT][NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      wp[nt] = w_ptr(ps, nt);
      const int co = min(co_w + 16 * nt + n, p.Cout - 1);
      const int32_t bv = p.bias ? p.bias[co] : 0;
      mc[nt] = p.m[co];
      sc[nt] = p.s[co];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = (v4i){bv, bv, bv, bv};
    }

    if (ps > 0) load_residual(co_w);   // pass 0: requested together with the activation tile

    // Software pipeline: the weights of chunk kk + 1 are requested before chunk kk is multiplied,
    // and the activation operand of the next 16-frame group is read from LDS while the current
    // one is multiplied.  The scheduling fences keep the compiler from sinking the requests
    // down to their first use.
    v4i wb[2][NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wb[0][nt] = *reinterpret_cast<const v4i*>(wp[nt]);
    v2i a0 = lds_read_tr8(abase + aoff[0]);
    v2i a1 = lds_read_tr8(abase + aoff[0] + 4096);

    for (int kc = 0; kc < ((g.dbg & 2) ? 0 : g.kch); kc += 2) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kk = kc + h;
        if (kk < g.kch) {
          const int kn = min(kk + 1, g.kch - 1);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            wb[h ^ 1][nt] = *reinterpret_cast<const v4i*>(wp[nt] + (int64_t)kn * 1024);
          __builtin_amdgcn_sched_barrier(0);
          const unsigned char* ab = abase + kk * 8192;
          const unsigned char* abn = abase + kn * 8192;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const v4i a = {a0.x, a0.y, a1.x, a1.y};
            const unsigned char* nx = (mt + 1 < MT) ? ab + aoff[mt + 1] : abn + aoff[0];
            a0 = lds_read_tr8(nx);
            a1 = lds_read_tr8(nx + 4096);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, wb[h][nt], acc[mt][nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }

    // ---- epilogue: lane (n, gi) holds frames 16 mt + 4 gi + (0..3) of channel co_w + 16 nt + n
    if (g.dbg & 4) continue;
    bool fast = true;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) fast = fast && sc[nt] >= 33;
    const bool all_fast = __all(fast);                  // wave-uniform: one code path
    if (p.res) {                                        // vmcnt(0): the residual tile is in LDS
      __builtin_amdgcn_s_waitcnt(0x0f70);
      asm volatile("" ::: "memory");
    }
    auto epilogue = [&](auto fast_tag, auto res_tag) {
      constexpr bool FAST = decltype(fast_tag)::value, RES = decltype(res_tag)::value;
      const int32_t hi127 = 127;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int sh = FAST ? sc[nt] - 32 : sc[nt], rnd = FAST ? 1 << (sc[nt] - 33) : 0;
        uint32_t rw[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          rw[mt] = RES ? *reinterpret_cast<const uint32_t*>(stage + nt * 2048 + soff[mt]) : 0u;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int32_t a4[4] = {acc[mt][nt][0], acc[mt][nt][1], acc[mt][nt][2], acc[mt][nt][3]};
          *reinterpret_cast<uint32_t*>(stage + nt * 2048 + soff[mt]) =
              requant_pack4<FAST, RES>(a4, mc[nt], sh, rnd, rw[mt], lo, hi127);
        }
      }
    };
    if (all_fast) {
      if (p.res) epilogue(std::true_type{}, std::true_type{}); else epilogue(std::true_type{}, std::false_type{});
    } else {
      if (p.res) epilogue(std::false_type{}, std::true_type{}); else epilogue(std::false_type{}, std::false_type{});
    }
    // rows out: lane -> (row 8 it + lane/8, slot lane%8) = unit u_l of channel co_w + row
#pragma unroll
    for (int it = 0; it < 2 * NT; ++it) {
      const v4i o = *reinterpret_cast<const v4i*>(stage + it * 1024 + lane * 16);
      const int co = co_w + 8 * it + (lane >> 3);
      if (u_ok && co < p.Cout) *reinterpret_cast<v4i*>(p.y + yoff_l + (int64_t)co * p.Tout) = o;
    }
  }
}

struct Choice { int MT, NT; };

size_t lds_bytes(const ConvParams& p, int NT) { return (size_t)p.Cin * 128 + (size_t)8 * 16 * NT * 128; }

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
  if (const char* e = getenv("QASR_PWT_MT")) {          // tuning override
    const int mt = atoi(e);
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
  g.dbg = 0;
  if (const char* e = getenv("QASR_PWT_DBG")) g.dbg = atoi(e);
  const size_t shmem = lds_bytes(p, NT);
  static bool attr_set = false;   // raise the dynamic LDS limit once per instantiation
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute((const void*)pw_tile_kernel<MT, NT>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles = (g.G + MT - 1) / MT;
  return launch_kernel(pw_tile_kernel<MT, NT>, dim3((unsigned)tiles), dim3(512), shmem, st, p, g);
}

}  // namespace

bool pw_tile_supported(const ConvParams& p) {
  if (p.depthwise || p.k != 1 || p.stride != 1 || p.pl != 0 || p.Tout != p.Tin) return false;
  if (!p.w_packed || p.Cin % 64 != 0 || p.Cin > 1024 || p.Tin % 16 != 0) return false;
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
