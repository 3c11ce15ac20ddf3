// Pointwise (k = 1) int8 convolution  Y[co, t] = sum_ci W[co, ci] * X[ci, t]  on the gfx950 int8
// matrix cores with the WEIGHTS stationary in registers, with the fused epilogue (bias, dyadic
// rescale, residual, clamp).
//
// At the batch sizes of the benchmark networks a layer has only a handful of 16-frame groups per
// compute unit, so how long ONE workgroup takes for its few groups is what a layer costs.  A
// workgroup of 8 waves owns up to 8 consecutive 16-frame groups (frames of all batch items, cut
// into groups of 16) and all input channels of them:
//
//   - the [Cin][16 * groups] activation tile comes into LDS once by direct global->LDS loads, rows
//     of 128 bytes with the 16-byte units XOR-swizzled (layout and transpose reads as in
//     pw_tile.hip), while
//   - wave w loads the weights of its 16*NT output channels for ALL input channels into registers
//     (KCH*NT operands of v_mfma_i32_16x16x64_i8, <= 128 VGPRs);
//   - then the wave walks group by group: the matrix products of group i (4*NT accumulators per
//     lane) are issued together with the epilogue arithmetic of group i - 1, which fills the issue
//     slots under the matrix pipeline; there are no barriers in this loop, so the two waves that
//     share a SIMD drift apart and overlap each other's stalls;
//   - int8 results are staged in a per-wave [16*NT][128 B] LDS tile (the residual tile was loaded
//     there up front) and leave as 64-byte row pieces, the first four groups as soon as they are
//     done, so that stores drain while the rest is still being multiplied.
//
// Requests are waited for in one go before the loop (the compiler's counters are exact there);
// the loop itself only stores.
#include "kernels.hpp"
#include "vmem.hpp"

#include <cstdlib>
#include <type_traits>

namespace qasr {

namespace {

typedef unsigned v4u __attribute__((ext_vector_type(4)));

struct PwsGeom {
  int G;          // 16-frame groups in total: B * Tin / 16
  int gpr;        // groups per row: Tin / 16
  int MT;         // groups per tile (<= 8)
  int tiles;      // ceil(G / MT)
  int per_xcd;    // tiles per XCD: ceil(tiles / 8)
  int co16n;      // ceil(Cout / 16)
};

__device__ __forceinline__ v2i lds_read_tr8(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr8_b64_v2i32(
      (v2i __attribute__((address_space(3)))*)(const_cast<unsigned char*>(p)));
}

template <int KCH, int NT>
__global__ __launch_bounds__(512) void pw_stream_kernel(ConvParams p, PwsGeom g) {
  extern __shared__ __align__(128) unsigned char lds[];  // [Cin][128] slots swizzled, then staging
  constexpr int ROWS = 16 * NT;                          // output channels of a wave

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, gi = lane >> 4;

  // Workgroup -> tile: consecutive workgroups go round-robin to the 8 XCDs (one L2 each);
  // neighbouring tiles share cache lines at their common edge, so each XCD gets a contiguous run.
  const int tile = (int)(blockIdx.x & 7) * g.per_xcd + (int)(blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= g.per_xcd || tile >= g.tiles) return;   // whole workgroup
  const int g0 = tile * g.MT;
  const int MT = min(g.MT, g.G - g0);                    // groups of this tile
  const int co_w = ((int)blockIdx.y * 8 + wave) * ROWS;  // wave-uniform
  const bool active = co_w < p.Cout;                     // idle waves still load and synchronise
  unsigned char* const stage = lds + KCH * 8192 + wave * (ROWS * 128);

  // ---- weights and per-channel constants -> registers (requested first: oldest)
  v4i w[KCH][NT];
  int32_t bv[NT], mc[NT], sc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int co16 = min((co_w >> 4) + nt, g.co16n - 1);
    const int8_t* wp = p.w + ((int64_t)co16 * KCH * 64 + lane) * 16;
#pragma unroll
    for (int kc = 0; kc < KCH; ++kc) w[kc][nt] = *reinterpret_cast<const v4i*>(wp + kc * 1024);
    const int co = min(co_w + 16 * nt + n, p.Cout - 1);
    bv[nt] = p.bias ? p.bias[co] : 0;
    mc[nt] = p.m[co];
    sc[nt] = p.s[co];
  }

  // ---- activation tile and residual tile: lane -> (row lane/8 of a block of 8 rows, slot lane%8);
  // the unit in that slot, slot ^ (row & 7), is the same for every block of 8 rows
  const int u_l = (lane & 7) ^ (lane >> 3);
  const int gq_l = g0 + u_l;
  const bool u_ok = u_l < MT;
  const int b_l = gq_l / g.gpr, t16_l = gq_l - b_l * g.gpr;
  const bool has_res = p.res != nullptr;
  if (has_res && active && u_ok) {
    const int8_t* src = p.res + (int64_t)b_l * p.ybs + 16 * t16_l;
#pragma unroll
    for (int it = 0; it < 2 * NT; ++it) {
      const int co = co_w + 8 * it + (lane >> 3);
      if (co < p.Cout) direct_load16(src + (int64_t)co * p.Tout, stage + it * 1024);
    }
  }
  if (u_ok) {
    const int8_t* src = p.x + (int64_t)b_l * p.xbs + (int64_t)(8 * wave + (lane >> 3)) * p.Tin + 16 * t16_l;
#pragma unroll
    for (int kc = 0; kc < KCH; ++kc)
      direct_load16(src + (int64_t)kc * 64 * p.Tin, lds + 8 * wave * 128 + kc * 8192);
  }

  // ---- per-lane constants of the transpose reads, the staging writes and the row stores.
  // Slot of unit mt in row r is mt ^ (r & 7): with the row's own (r & 7) << 4 folded into the
  // lane's base offset, the address of unit mt is base ^ (mt << 4).
  const int l16 = lane & 15, j = l16 >> 1;
  const uint32_t abase = (uint32_t)((8 * gi + j) * 128 + 8 * (l16 & 1)) | (uint32_t)(j << 4);
  const uint32_t sbase = (uint32_t)(n * 128 + 4 * gi) | (uint32_t)((n & 7) << 4);   // stage row 16 nt + n
  const int lo = p.relu ? 0 : -128;
  const int32_t hi127 = 127;
  // Row stores: lane -> (row lane/4 of a block of 16 rows, unit lane%4 of the first four, or
  // 4 + lane%4 of the rest).  Offsets of lanes without a row or a unit are rejected by the resource.
  const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
      p.y + (int64_t)co_w * p.Tout, 0, 0x7ffffff0, 0x00027000);
  uint32_t y_off[2];
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
    const int u = 4 * hf + (lane & 3), gq = g0 + u;
    const int b = gq / g.gpr, t16 = gq - b * g.gpr;
    y_off[hf] = u < MT ? (uint32_t)b * (uint32_t)p.ybs + 16u * (uint32_t)t16 + (uint32_t)(lane >> 2) * (uint32_t)p.Tout
                       : 0xfffffff0u;
  }

  // everything requested so far has arrived; the other waves' rows too
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
    for (int kc = 0; kc < KCH; ++kc) tie(w[kc][nt]);
    tie(bv[nt]); tie(mc[nt]); tie(sc[nt]);
  }
  wait_vm<0>();
  __syncthreads();
  if (!active) return;

  bool fast = true;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) fast = fast && sc[nt] >= 33;
  const bool all_fast = __all(fast);                  // wave-uniform: one epilogue variant

  // rows out for units 4 hf .. 4 hf + 3
  auto store_half = [&](int hf) {
#pragma unroll
    for (int it = 0; it < NT; ++it) {
      const int row = 16 * it + (lane >> 2);
      const int slot = (4 * hf + (lane & 3)) ^ (row & 7);
      const v4i o = *reinterpret_cast<const v4i*>(stage + row * 128 + slot * 16);
      const bool ok = co_w + row < p.Cout;
      __builtin_amdgcn_raw_buffer_store_b128((v4u){(unsigned)o.x, (unsigned)o.y, (unsigned)o.z, (unsigned)o.w}, yrs,
                                             ok && y_off[hf] != 0xfffffff0u ? y_off[hf] + (uint32_t)(16 * it) * (uint32_t)p.Tout
                                                                            : 0xfffffff0u, 0, 0);
    }
  };

  // One step = the matrix products of group i (accumulators i % 2) together with the epilogue of
  // group i - 1 (accumulators (i - 1) % 2): lane (n, gi) holds frames 4 gi + (0..3) of channel
  // co_w + 16 nt + n.
  v4i acc[2][NT];
  // CUR: group i is multiplied; PREV: group i - 1 gets its epilogue.  Both are compile-time so that
  // the body is one straight-line block, in which the scheduling groups below pin the order
  //   LDS reads | (1 matrix product, 6 vector ops) x NT | LDS write
  // for the chunk steps that carry an epilogue column: the wave issues in order, so only vector
  // work placed between two matrix products runs under the first one.
  auto step = [&](int i, int par, auto fast_tag, auto res_tag, auto cur_tag, auto prev_tag) {
    constexpr bool FAST = decltype(fast_tag)::value, RES = decltype(res_tag)::value;
    constexpr bool CUR = decltype(cur_tag)::value, PREV = decltype(prev_tag)::value;
    if (CUR) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[par][nt] = (v4i){bv[nt], bv[nt], bv[nt], bv[nt]};
    }
    const unsigned char* ab = lds + (abase ^ (uint32_t)(i << 4));
    unsigned char* const st = stage + (sbase ^ ((((uint32_t)i + 7u) & 7u) << 4));   // unit i - 1
#pragma unroll
    for (int kc = 0; kc < KCH; ++kc) {
      const bool epi = PREV && kc < NT;         // one 16-channel column of the previous group
      if (CUR) {
        const v2i a0 = lds_read_tr8(ab + kc * 8192);
        const v2i a1 = lds_read_tr8(ab + kc * 8192 + 4096);
        const v4i a = {a0.x, a0.y, a1.x, a1.y};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[par][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, w[kc][nt], acc[par][nt], 0, 0, 0);
      }
      if (epi) {
        const int nt = kc;
        const int sh = FAST ? sc[nt] - 32 : sc[nt], rnd = FAST ? 1 << (sc[nt] - 33) : 0;
        uint32_t* const sp = reinterpret_cast<uint32_t*>(st + nt * 2048);
        const uint32_t rw = RES ? *sp : 0u;
        const v4i av = acc[par ^ 1][nt];
        const int32_t a4[4] = {av[0], av[1], av[2], av[3]};
        *sp = requant_pack4<FAST, true>(a4, mc[nt], sh, rnd, rw, lo, hi127);
      }
      if (CUR && FAST) {
        if (epi && RES) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);            // LDS reads
        else __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          // matrix product
          if (epi) __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);                 // vector ops
        }
        if (epi) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                   // LDS write
      }
    }
    if (i == 4) store_half(0);                 // groups 0..3 are staged
  };
  auto run = [&](auto fast_tag, auto res_tag) {
    const std::true_type T{};
    const std::false_type F{};
    step(0, 0, fast_tag, res_tag, T, F);
    int i = 1;
    for (; i + 1 < MT; i += 2) {
      step(i, 1, fast_tag, res_tag, T, T);
      step(i + 1, 0, fast_tag, res_tag, T, T);
    }
    if (i < MT) { step(i, 1, fast_tag, res_tag, T, T); ++i; }
    step(i, i & 1, fast_tag, res_tag, F, T);   // i == MT: the last group's epilogue
  };
  if (all_fast) {
    if (has_res) run(std::true_type{}, std::true_type{}); else run(std::true_type{}, std::false_type{});
  } else {
    if (has_res) run(std::false_type{}, std::true_type{}); else run(std::false_type{}, std::false_type{});
  }
  if (MT < 4) store_half(0);                   // (not reached inside the loop)
  if (MT > 4) store_half(1);
}

struct Choice { int KCH, NT, splits; };

// activation tile + per-wave staging
size_t lds_bytes(int KCH, int NT) { return (size_t)KCH * 8192 + (size_t)8 * 16 * NT * 128; }

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
bool pick(const ConvParams& p, Choice& c) {
  if (getenv("QASR_NO_PW_STREAM")) return false;          // tuning: fall through to pw_tile
  if (p.depthwise || p.k != 1 || p.stride != 1 || p.pl != 0 || p.Tout != p.Tin) return false;
  if (!p.w_packed || p.Tin % 16 != 0 || p.Cin % 64 != 0) return false;
  if (p.xbs % 16 != 0 || p.ybs % 16 != 0) return false;
  if ((uintptr_t)p.x % 16 || (uintptr_t)p.y % 16 || (uintptr_t)p.w % 16 || (p.res && (uintptr_t)p.res % 16))
    return false;
  if ((int64_t)p.B * p.ybs >= 0x7ffffff0LL) return false;          // 32-bit output offsets
  if ((int64_t)p.B * (p.Tin / 16) > 0x3fffffff) return false;
  c.KCH = p.Cin / 64;
  // instantiated (KCH, NT) pairs: KCH * NT operands of 4 registers each stay resident
  if (c.KCH == 4) c.NT = p.Cout > 256 ? 4 : 2;
  else if (c.KCH == 8) c.NT = 4;
  else return false;
  if (p.Cout < 64 * c.NT) return false;                 // too few output channels for 8 waves
  c.splits = (p.Cout + 128 * c.NT - 1) / (128 * c.NT);
  if (c.splits > 65535) return false;
  return lds_bytes(c.KCH, c.NT) <= 160 * 1024;
}

template <int KCH, int NT>
hipError_t launch_t(const ConvParams& p, const Choice& c, hipStream_t st) {
  PwsGeom g;
  g.gpr = p.Tin / 16;
  g.G = p.B * g.gpr;
  g.co16n = (p.Cout + 15) / 16;
  // groups per tile: least makespan over the CUs (one workgroup per CU at a time; the output-channel
  // splits share them), with a per-tile overhead worth about two groups
  const int cus = num_cus();
  double best = 1e300;
  g.MT = 8;
  for (int MT = 3; MT <= 8; ++MT) {
    const int64_t wgs = (int64_t)((g.G + MT - 1) / MT) * c.splits;
    const double cost = (double)((wgs + cus - 1) / cus) * (MT + 2.0);
    if (cost < best - 1e-9) { best = cost; g.MT = MT; }
  }
  if (const char* e = getenv("QASR_PWS_MT")) {           // tuning override
    const int v = atoi(e);
    if (v >= 1 && v <= 8) g.MT = v;
  }
  g.tiles = (g.G + g.MT - 1) / g.MT;
  g.per_xcd = (g.tiles + 7) / 8;
  const size_t shmem = lds_bytes(KCH, NT);
  static bool attr_set = false;   // raise the dynamic LDS limit once per instantiation
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute((const void*)pw_stream_kernel<KCH, NT>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  return launch_kernel(pw_stream_kernel<KCH, NT>, dim3((unsigned)(8 * g.per_xcd), (unsigned)c.splits),
                       dim3(512), shmem, st, p, g);
}

}  // namespace

bool pw_stream_supported(const ConvParams& p) {
  Choice c;
  return pick(p, c);
}

hipError_t launch_pw_stream(const ConvParams& p, hipStream_t st) {
  Choice c;
  if (!pick(p, c)) return hipErrorInvalidValue;
  if (c.KCH == 4 && c.NT == 2) return launch_t<4, 2>(p, c, st);
  if (c.KCH == 4 && c.NT == 4) return launch_t<4, 4>(p, c, st);
  if (c.KCH == 8 && c.NT == 4) return launch_t<8, 4>(p, c, st);
  return hipErrorInvalidValue;
}

}  // namespace qasr
