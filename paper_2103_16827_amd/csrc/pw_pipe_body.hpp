// One tile of the pipelined pointwise kernel as a device function: called by the stand-alone kernel
// (pw_pipe.hip, one tile per workgroup) and by the persistent team kernel (team.hip, which walks a
// list of layers with barriers among the workgroups of an XCD in between).  See pw_pipe.hip for
// what the tile does.
#pragma once
#include "common.hpp"
#include "vmem.hpp"

#include <type_traits>

namespace qasr {
namespace pwp {

typedef unsigned v4u __attribute__((ext_vector_type(4)));

// cache policy of the output stores (sc0 sc1): written through towards memory as they are issued,
// so that little is left to write back when the kernel ends
constexpr int kStoreThrough = 17;
constexpr int NT = 2;           // 16-channel columns per wave and pass
constexpr int ROWS = 16 * NT;   // output channels of a wave and pass
constexpr int kLookW = 4;       // weight chunks requested ahead of the one being multiplied (the stand-alone kernel)
constexpr int LOOKX = 3;        // activation chunks requested ahead in pass 0
constexpr int kMaxMT = 7;       // groups per tile: two accumulator sets of 8 groups would not fit the registers
constexpr int MAXP = 8;         // passes (Cout <= 2048): bounds the constants parked in LDS

struct PwpGeom {
  int G;        // 16-frame groups in total: B * Tin / 16
  int gpr;      // groups per row: Tin / 16
  int passes;   // ceil(Cout / 256)
  int co16n;    // ceil(Cout / 16)
  int tiles, tiles_per_xcd;
  int splits, pps;   // workgroups per tile (each takes pps consecutive passes of the output channels)
  int nopipe;        // tuning: every pass does its epilogue right after its own products
};

__device__ __forceinline__ v2i lds_read_tr8(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr8_b64_v2i32(
      (v2i __attribute__((address_space(3)))*)(const_cast<unsigned char*>(p)));
}

// LDS: [XCH * 64 rows][128 B]  activation tile (unit u of row r in slot u ^ (r & 7)); XCH = KCH up to
//      512 input channels: the whole tile stays; beyond that a ring of 8 chunks (chunk kc in slot
//      kc & 7) that the single pass of the workgroup streams through
//      [8 waves][2][ROWS][128 B] staging: residual rows in, int8 rows out, per wave and pass parity
//      [8 waves][MAXP][NT][3][16] dwords: bias, m, s of the wave's channels of every pass
//      [8 waves][256 B] the fused activation's table (one copy per wave: no barrier needed)
template <int KCH>
constexpr int lds_bytes_c() { return (KCH < 8 ? KCH : 8) * 8192 + 8 * 2 * ROWS * 128 + 8 * MAXP * NT * 3 * 64 + 8 * 256; }
// The lean form (see LEAN below): the activation tile and one 16-row staging block per wave, which
// also holds the wave's constants until the epilogue starts; at 512 input channels exactly half
// of a compute unit's LDS, so that two workgroups are resident together.
// Residual rows (4 KiB per wave) have an area of their own after the staging blocks at 256 input
// channels; at 512 there is no room left, and they land in the LDS of the first four activation
// chunks once every wave is done with those (see the chunk loop).
template <int KCH>
constexpr int lds_bytes_lean_c() { return (KCH < 8 ? KCH : 8) * 8192 + 8 * 16 * 128 + (KCH < 8 ? 8 * 4096 : 0); }
constexpr int kLeanResAfter = 5;   // 512 input channels: residual rows requested behind the barrier of chunk step 5

// ACT: a unary activation's table is applied after the clamp (an instantiation of its own: the
// plain layers keep their code as it is)
// TEAM: the tile runs inside the persistent team kernel: `vblock` is the tile itself (no XCD
// interleave, no pass split), activations and residual rows were written earlier in the same kernel
// by other workgroups of this XCD, so they are loaded at device scope (past the vector cache, out of
// the XCD's L2), and the output rows are stored write-back (the next layer reads them from that L2).
// LOOK: weight chunks requested ahead of the one being multiplied (a ring of LOOK x NT x 4 registers).
// LEAN: exactly one pass per workgroup (the launcher gives every pass of a tile a workgroup of its
// own), one accumulator set, no fused activation, staging of 16 rows at a
// time: half the registers and half the LDS, so that two workgroups share a compute unit and each
// SIMD has four waves to pick instructions from; the epilogue of one workgroup then overlaps the
// products of the other by chance instead of by construction.
template <int MT, int KCH, bool ACT, bool TEAM, int LOOK = kLookW, bool LEAN = false>
__device__ __forceinline__ void pw_pipe_tile(const ConvParams& p, const PwpGeom& g, unsigned vblock,
                                             unsigned char* const xs, int tid) {
  constexpr int NB = MT * NT;                     // epilogue blocks of a pass
  static_assert(KCH == 4 || KCH == 8 || KCH == 16 || KCH == 32, "instantiated input widths");
  static_assert(KCH % LOOK == 0, "ring slot of a chunk");
  static_assert(!LEAN || (!ACT && !TEAM && KCH <= 8), "the lean form: plain layers, resident tile");

  // `tid`: the thread's index in the workgroup (threadIdx.x).
  // (inside the team kernel's layer loop: keeps everything derived from the thread id inside the
  // tile, or the compiler computes the lane constants of every layer body once, ahead of the loop,
  // and has to carry them through all the bodies in registers that do not exist)
  if constexpr (TEAM) asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, gi = lane >> 4;
  // Workgroup -> tile: consecutive workgroups go round-robin to the 8 XCDs (one L2 each);
  // neighbouring tiles share the cache lines at their common edge, so each XCD gets a contiguous run.
  // When the tiles alone do not fill the chip, `splits` workgroups share a tile, each with its own
  // run of passes (the tile's workgroups have the same blockIdx & 7: same XCD, the activation tile
  // comes out of that L2 for all but the first).
  const int bx = TEAM ? (int)vblock : (int)(vblock % (unsigned)(8 * g.tiles_per_xcd));
  const int pb = TEAM ? 0 : (int)(vblock / (unsigned)(8 * g.tiles_per_xcd)) * g.pps;     // first pass of this workgroup
  const int tile = TEAM ? bx : (bx & 7) * g.tiles_per_xcd + (bx >> 3);
  if (tile >= g.tiles) return;                                                     // whole workgroup
  const int g0 = tile * MT;
  // passes in which this wave has channels (>= 1: Cout >= 256, and a multiple of 256 when split);
  // it leaves after them
  const int P = LEAN ? 1 : min(g.pps, min(g.passes, (p.Cout - wave * ROWS + 8 * ROWS - 1) / (8 * ROWS)) - pb);

  // lane -> (row lane/8 of a block of 8 rows, slot lane%8); the unit in that slot, slot ^ (row & 7),
  // is the same for every block of 8 rows: one lane -> unit map for activation loads, residual
  // loads and output stores.
  const int u_l = (lane & 7) ^ (lane >> 3);
  const int gq_l = g0 + u_l;
  const bool u_ok = u_l < MT && gq_l < g.G;
  const int b_l = gq_l / g.gpr, t16_l = gq_l - b_l * g.gpr;
  const int64_t yoff_l = (int64_t)b_l * p.ybs + 16 * t16_l;       // of this lane's unit
  constexpr int XCH = KCH < 8 ? KCH : 8;          // activation chunks resident in LDS
  unsigned char* const stage0 = xs + XCH * 8192 + wave * (LEAN ? 16 * 128 : 2 * ROWS * 128);
  // (lean: the constants of the one pass sit in the wave's staging block, 384 of its 2048 bytes, and
  // are all in registers before the first staged word is written)
  unsigned char* const cst0 = LEAN ? stage0 : xs + XCH * 8192 + 8 * 2 * ROWS * 128 + wave * (MAXP * NT * 3 * 64);
  const bool has_res = p.res != nullptr;
  // (lean: where the wave's residual rows land, [NT][16 rows][128 B])
  unsigned char* const lres0 = KCH < 8 ? xs + XCH * 8192 + 8 * 16 * 128 + wave * 4096 : xs + wave * 4096;
  unsigned char* const lutw = xs + XCH * 8192 + 8 * 2 * ROWS * 128 + 8 * (MAXP * NT * 3 * 64) + wave * 256;
  constexpr bool has_act = ACT;                     // a unary activation follows the clamp

  int seq = 0;                                   // vector-memory requests issued by this wave
  int mark_r[2] = {0, 0}, mark_c = 0, mark_w[LOOK] = {}, mark_x[KCH] = {};

  auto issue_residual = [&](int ps, int par) __attribute__((always_inline)) {   // residual rows of pass ps -> stage[par]
    if (has_res) {
      const int co_w = ((pb + ps) * 8 + wave) * ROWS;
      unsigned char* const dst = LEAN ? lres0 : stage0 + par * (ROWS * 128);
#pragma unroll
      for (int it = 0; it < 2 * NT; ++it) {
        const int co = co_w + 8 * it + (lane >> 3);
        if (u_ok && co < p.Cout)
          direct_load16_scope<TEAM>(p.res + yoff_l + (int64_t)co * p.Tout, dst + it * 1024);
        if (co_w + 8 * it < p.Cout) ++seq;       // issued iff some lane had a row (lane 0 has unit 0)
      }
    }
    mark_r[par] = seq;
  };
  // weight stream: the chunks of the wave's passes in order; past the last pass it goes on with
  // that pass's first chunks again (in bounds, never multiplied)
  const v4i wrsrc = make_rsrc(p.w, (uint32_t)g.co16n * (uint32_t)KCH * 1024u);
  const uint32_t wlane = (uint32_t)lane * 16;
  v4i wb[LOOK][NT];                               // ring of weight chunks, LOOK chunks ahead of the products
  // byte offset of chunk 0 of the wave's block nt in pass ps (wave-uniform)
  auto pass_base = [&](int ps, int nt) __attribute__((always_inline)) {
    const int co16 = min(((pb + min(ps, P - 1)) * 8 + wave) * NT + nt, g.co16n - 1);
    return (uint32_t)__builtin_amdgcn_readfirstlane(co16 * (KCH * 1024));
  };
  auto issue_w = [&](const uint32_t (&base)[NT], int kc, int h) __attribute__((always_inline)) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wb[h][nt] = bload16(wrsrc, wlane, base[nt] + (uint32_t)kc * 1024u);
    seq += NT;
    mark_w[h] = seq;
  };
  uint32_t wcur[NT], wnext[NT];                   // pass_base of the pass being multiplied and of the one after
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) { wcur[nt] = pass_base(0, nt); wnext[nt] = pass_base(1, nt); }

  // ---- requests of the start: residual of pass 0, constants of all passes, then the first weight
  // and activation chunks (the first products need only 64 channels)
  if (!LEAN || KCH < 8) issue_residual(0, 0);
  for (int ps = 0; ps < P; ++ps) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int co = min(((pb + ps) * 8 + wave) * ROWS + 16 * nt + n, p.Cout - 1);
      unsigned char* d = cst0 + (ps * NT + nt) * (3 * 64);
      if (lane < 16) {
        if (p.bias) direct_load4(p.bias + co, d);
        direct_load4(p.m + co, d + 64);
        direct_load4(p.s + co, d + 128);
      }
      seq += p.bias ? 3 : 2;
    }
  }
  if (has_act) {                                   // 64 lanes x 4 bytes: the wave's copy of the table
    direct_load4(p.act_lut + 4 * lane, lutw);
    ++seq;
  }
  mark_c = seq;
  // Activation chunk kc of this wave: rows 64 kc + 8 wave + (0..7).  Only the first LOOKX chunks are
  // requested here, chunk kc + LOOKX during chunk step kc of pass 0: all workgroups start
  // together, and a request waits behind everything that entered the memory system before it,
  // so what is multiplied first has to be asked for first chip-wide.
  const int8_t* const xsrc = p.x + (int64_t)b_l * p.xbs + (int64_t)(8 * wave + (lane >> 3)) * p.Tin + 16 * t16_l;
  const int64_t xstep = (int64_t)64 * p.Tin;
  auto issue_x = [&](int kc) __attribute__((always_inline)) {
    if (u_ok) direct_load16_scope<TEAM>(xsrc + kc * xstep, xs + 8 * wave * 128 + (kc & 7) * 8192);
    mark_x[kc] = ++seq;
  };
  issue_w(wcur, 0, 0);
  issue_x(0);
  issue_w(wcur, 1, 1);
  issue_x(1);
#pragma unroll
  for (int q = 2; q < LOOK; ++q) issue_w(wcur, q, q);
#pragma unroll
  for (int kc = 2; kc < LOOKX && kc < KCH; ++kc) issue_x(kc);

  // per-lane constants of the transpose reads, staging accesses and row stores (see pw_tile.hip)
  const int l16 = lane & 15, j = l16 >> 1;
  const uint32_t abase = (uint32_t)((8 * gi + j) * 128 + 8 * (l16 & 1)) | (uint32_t)(j << 4);
  const uint32_t sbase = (uint32_t)(n * 128 + 4 * gi) | (uint32_t)((n & 7) << 4);   // stage row 16 nt + n
  const int lo = p.relu ? 0 : -128;
  const int32_t hi127 = 127;
  const uint32_t y_lane = u_ok ? (uint32_t)yoff_l + (uint32_t)(lane >> 3) * (uint32_t)p.Tout : 0xfffffff0u;

  v4i acc[LEAN ? 1 : 2][MT][NT];
  int32_t mc[NT], sh[NT], rnd[NT];                // rescale constants of the pass whose epilogue is pending

  // one epilogue block: lane (n, gi) holds frames 16 mt + 4 gi + (0..3) of channel 16 nt + n
  auto block = [&](int par, int e, auto fast_tag, auto res_tag) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast_tag)::value, RES = decltype(res_tag)::value;
    const int mt = e / NT, nt = e % NT;
    uint32_t* const sp = reinterpret_cast<uint32_t*>(stage0 + (LEAN ? 0 : par * (ROWS * 128) + nt * 2048) + (sbase ^ (uint32_t)(mt << 4)));
    const uint32_t rw = !RES ? 0u : LEAN ? *reinterpret_cast<const uint32_t*>(lres0 + nt * 2048 + (sbase ^ (uint32_t)(mt << 4))) : *sp;
    const v4i av = acc[par][mt][nt];
    const int32_t a4[4] = {av[0], av[1], av[2], av[3]};
    uint32_t pk = requant_pack4<FAST, RES>(a4, mc[nt], sh[nt], rnd[nt], rw, lo, hi127);
    if (has_act) {                                 // table[code + 128], byte by byte
      const uint32_t c = pk ^ 0x80808080u;
      pk = (uint32_t)lutw[c & 0xffu] | ((uint32_t)lutw[(c >> 8) & 0xffu] << 8) |
           ((uint32_t)lutw[(c >> 16) & 0xffu] << 16) | ((uint32_t)lutw[c >> 24] << 24);
    }
    *sp = pk;
  };
  // The pipelined case (short-form rescale, relu): the epilogue of a pass is a stream of 4 NB
  // "elements" (element x = accumulator register x % 4 of block x / 4), each going through six
  // one-instruction stages
  //   S0 h = mulhi(acc, m)   S1 h += rnd   S2 h >>= sh   S3 h += residual byte   S4 h = clamp(h, 0, 127)
  //   S5 pack into the block's word (and write the word to the staging tile after the 4th element)
  // Element x enters at step 2x and advances one stage per step, so step t carries three
  // instructions that belong to three different elements and do not depend on each other; what
  // an instruction needs was produced at least one matrix product earlier.  One step rides on
  // every product of the following pass (two when Cin = 256); the last five steps follow the loop.
  // The residual word of block e + 1 is read while block e is in flight.
  constexpr int NE = 4 * NB;                      // elements of a pass
  constexpr int NSTEPS = 2 * NE + 4;              // steps 0 .. 2 (NE - 1) + 5
  int32_t ph[3] = {0, 0, 0};                      // element x lives in ph[x % 3]
  uint32_t pword = 0, rw[2] = {0u, 0u};           // pack word of the block at S5; residual word of block e in rw[e & 1]
  auto stage_word = [&](int par, int e) __attribute__((always_inline)) {
    const int mt = e / NT, nt = e % NT;
    return reinterpret_cast<uint32_t*>(stage0 + par * (ROWS * 128) + nt * 2048 + (sbase ^ (uint32_t)(mt << 4)));
  };
  // (RES false: no residual byte is added at S3; the stages stay the same)
  auto step = [&](int par, int t, auto res_tag) __attribute__((always_inline)) {
    constexpr bool RES = decltype(res_tag)::value;
    const int x0 = t >> 1, x1 = x0 - 1, x2 = x0 - 2;        // the elements at stages (S0|S1), (S2|S3), (S4|S5)
    if ((t & 1) == 0) {
      if (x0 < NE) {
        const int e = x0 >> 2, i = x0 & 3;
        ph[x0 % 3] = mulhi_i32(acc[par][e / NT][e % NT][i], mc[e % NT]);
        if (RES && i == 1 && e + 1 < NB) rw[(e + 1) & 1] = *stage_word(par, e + 1);
      }
      if (x1 >= 0 && x1 < NE) ph[x1 % 3] >>= sh[(x1 >> 2) % NT];
      if (x2 >= 0 && x2 < NE) ph[x2 % 3] = min(max(ph[x2 % 3], 0), 127);
    } else {
      if (x0 < NE) ph[x0 % 3] += rnd[(x0 >> 2) % NT];
      if (RES && x1 >= 0 && x1 < NE) ph[x1 % 3] += (int32_t)(int8_t)(rw[(x1 >> 2) & 1] >> (8 * (x1 & 3)));
      if (x2 >= 0 && x2 < NE) {
        const int e = x2 >> 2, i = x2 & 3;
        pword = i == 0 ? (uint32_t)ph[x2 % 3] : (pword | ((uint32_t)ph[x2 % 3] << (8 * i)));
        if (i == 3) *stage_word(par, e) = pword;
      }
    }
  };
  // rows of pass ps out of stage[par]: lane -> (row 8 it + lane/8, slot lane%8)
  auto store_rows = [&](int ps, int par) __attribute__((always_inline)) {
    const int co_w = ((pb + ps) * 8 + wave) * ROWS;
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
        p.y + (int64_t)co_w * p.Tout, 0, 0x7ffffff0, 0x00027000);
#pragma unroll
    for (int it = 0; it < 2 * NT; ++it) {
      const v4i o = *reinterpret_cast<const v4i*>(stage0 + par * (ROWS * 128) + it * 1024 + lane * 16);
      const bool ok = u_ok && co_w + 8 * it + (lane >> 3) < p.Cout;
      const v4u ov = {(unsigned)o.x, (unsigned)o.y, (unsigned)o.z, (unsigned)o.w};
      const uint32_t off = ok ? y_lane + (uint32_t)(8 * it) * (uint32_t)p.Tout : 0xfffffff0u;
      __builtin_amdgcn_raw_buffer_store_b128(ov, yrs, off, 0, TEAM ? 0 : kStoreThrough);
    }
  };
  // lean: the 16 rows of column block nt out of the wave's one staging block
  auto store_rows_lean = [&](int ps, int nt) __attribute__((always_inline)) {
    const int co_w = ((pb + ps) * 8 + wave) * ROWS;
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
        p.y + (int64_t)co_w * p.Tout, 0, 0x7ffffff0, 0x00027000);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int it = 2 * nt + h;
      const v4i o = *reinterpret_cast<const v4i*>(stage0 + h * 1024 + lane * 16);
      const bool ok = u_ok && co_w + 8 * it + (lane >> 3) < p.Cout;
      const v4u ov = {(unsigned)o.x, (unsigned)o.y, (unsigned)o.z, (unsigned)o.w};
      const uint32_t off = ok ? y_lane + (uint32_t)(8 * it) * (uint32_t)p.Tout : 0xfffffff0u;
      __builtin_amdgcn_raw_buffer_store_b128(ov, yrs, off, 0, kStoreThrough);
    }
  };
  constexpr int STORE_REQS = 2 * NT;              // requests of one store_rows
  // the epilogue of pass ps on its own
  auto epilogue_alone = [&](int ps, int par, auto fast_tag) __attribute__((always_inline)) {
    if constexpr (LEAN) {
      if (has_res) wait_vm_dyn(seq - mark_r[0]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if (has_res) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            block(par, mt * NT + nt, fast_tag, std::true_type{});
            if (mt & 1) __builtin_amdgcn_sched_barrier(0);
          }
        } else {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            block(par, mt * NT + nt, fast_tag, std::false_type{});
            if (mt & 1) __builtin_amdgcn_sched_barrier(0);
          }
        }
        store_rows_lean(ps, nt);
      }
      seq += STORE_REQS;
      return;
    }
    if (has_res) wait_vm_dyn(seq - mark_r[par]);          // residual rows of this pass
    if (has_res) {
#pragma unroll
      for (int e = 0; e < NB; ++e) {
        block(par, e, fast_tag, std::true_type{});
        if (e & 1) __builtin_amdgcn_sched_barrier(0);       // bounds the live temporaries
      }
    } else {
#pragma unroll
      for (int e = 0; e < NB; ++e) {
        block(par, e, fast_tag, std::false_type{});
        if (e & 1) __builtin_amdgcn_sched_barrier(0);
      }
    }
    store_rows(ps, par);
    seq += STORE_REQS;
  };

  bool pending = false;       // the pass before awaits its (short-form) epilogue
  // The multiply loop of pass ps into accumulator set par; PREV: the epilogue of pass ps - 1 rides along.
  // (FIRST: pass 0, which also waits for the activation chunks and synchronises the waves)
  auto multiply = [&](int ps, int par, auto prev_tag, auto first_tag, auto res_tag) __attribute__((always_inline)) {
    constexpr bool PREV = decltype(prev_tag)::value, FIRST = decltype(first_tag)::value, RES = decltype(res_tag)::value;
    // bias of this pass out of LDS (constants of all passes were requested at the start)
    if (FIRST) wait_vm_dyn(seq - mark_c);
    if (!FIRST) issue_residual(ps, par);      // stage[par] is free: its rows left at the end of pass ps - 1
    if (!FIRST) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) { wcur[nt] = wnext[nt]; wnext[nt] = pass_base(ps + 1, nt); }
    }
    {
      const unsigned char* c = cst0 + ps * (NT * 3 * 64) + 4 * n;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int32_t bv = p.bias ? *reinterpret_cast<const int32_t*>(c + nt * 192) : 0;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[par][mt][nt] = (v4i){bv, bv, bv, bv};
      }
    }
    if (PREV) {
      if (RES) wait_vm_dyn(seq - mark_r[par ^ 1]);          // residual rows of the pass before
      if (RES) rw[0] = *stage_word(par ^ 1, 0);
    }

#pragma unroll
    for (int kk = 0; kk < KCH; ++kk) {
      const int h = kk % LOOK;                    // KCH is a multiple of LOOK: the ring restarts per pass
      // weights of this chunk and, in pass 0, the activation chunk(s) needed so far
      if (FIRST) {
        {
          const int mw = mark_w[h], mx = mark_x[kk];   // (by value: no references to the marks)
          wait_vm_dyn(seq - (mw > mx ? mw : mx));
        }
      } else if (kk < LOOK) {
        wait_vm_dyn(seq - mark_w[h]);
      } else {
        wait_vm<(LOOK - 1) * NT>();               // only the following chunks' weights are younger
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) tie(wb[h][nt]);
      if (FIRST) {
        __syncthreads();                          // publishes the other waves' rows of the chunk
        if (kk + LOOKX < KCH) issue_x(kk + LOOKX);
        // lean, 512 input channels: behind this barrier every wave has read the chunks before
        // kk - 1 for the last time, so from step 5 on the LDS of chunks 0..3 can take the residual rows
        if (LEAN && KCH == 8 && kk == kLeanResAfter) issue_residual(0, 0);
      }
      {
        const unsigned char* ab = xs + (kk & 7) * 8192;
        // the operand of group mt + 2 is read while groups mt and mt + 1 are multiplied
        v2i ar[3][2];
#pragma unroll
        for (int q = 0; q < 2 && q < MT; ++q) {
          ar[q][0] = lds_read_tr8(ab + (abase ^ (uint32_t)(q << 4)));
          ar[q][1] = lds_read_tr8(ab + (abase ^ (uint32_t)(q << 4)) + 4096);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const v4i a = {ar[mt % 3][0].x, ar[mt % 3][0].y, ar[mt % 3][1].x, ar[mt % 3][1].y};
          if (mt + 2 < MT) {
            ar[(mt + 2) % 3][0] = lds_read_tr8(ab + (abase ^ (uint32_t)((mt + 2) << 4)));
            ar[(mt + 2) % 3][1] = lds_read_tr8(ab + (abase ^ (uint32_t)((mt + 2) << 4)) + 4096);
          }
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            acc[par][mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, wb[h][nt], acc[par][mt][nt], 0, 0, 0);
            if (PREV) {
              constexpr int R = KCH <= 8 ? 8 / KCH : 0;   // steps per product: 8 NB steps over KCH MT NT products
              const int slot = (kk * MT + mt) * NT + nt;
#pragma unroll
              for (int r = 0; r < R; ++r) step(par ^ 1, slot * R + r, res_tag);
              __builtin_amdgcn_sched_barrier(0);  // one product, its epilogue steps, nothing else
            }
          }
          if (!PREV) __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (kk + LOOK < KCH) issue_w(wcur, kk + LOOK, h);
      else issue_w(wnext, kk + LOOK - KCH, h);
    }
    if (PREV) {
#pragma unroll
      for (int t = 8 * NB; t < NSTEPS; ++t) step(par ^ 1, t, res_tag);     // the last elements drain
      store_rows(ps - 1, par ^ 1);                 // (the caller counts these requests)
    }
  };
  // One pass: multiply, then either leave the epilogue pending for the next pass (short-form
  // rescale and a next pass exists) or do it now.
  auto do_pass = [&](int ps, int par, auto first_tag) __attribute__((always_inline)) {
    const std::true_type T{};
    const std::false_type F{};
    if (decltype(first_tag)::value) multiply(ps, par, F, T, F);
    else if (pending && has_res) multiply(ps, par, T, F, T);
    else if (pending) multiply(ps, par, T, F, F);
    else multiply(ps, par, F, F, F);
    seq += pending ? STORE_REQS : 0;      // rows of the pass before, stored at the end of the loop
    // rescale constants of this pass
    const unsigned char* c = cst0 + ps * (NT * 3 * 64) + 4 * n;
    bool fast = true;
    int32_t s_[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      mc[nt] = *reinterpret_cast<const int32_t*>(c + nt * 192 + 64);
      s_[nt] = *reinterpret_cast<const int32_t*>(c + nt * 192 + 128);
      fast = fast && s_[nt] >= 33;
    }
    const bool all_fast = __builtin_amdgcn_readfirstlane((int)__all(fast)) != 0;   // wave-uniform, and known to be
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      sh[nt] = all_fast ? s_[nt] - 32 : s_[nt];
      rnd[nt] = all_fast ? 1 << ((s_[nt] - 33) & 31) : 0;
    }
    if (all_fast && p.relu && !has_act && ps + 1 < P && !g.nopipe) {
      pending = true;
    } else {
      pending = false;
      if (all_fast) epilogue_alone(ps, par, std::true_type{}); else epilogue_alone(ps, par, std::false_type{});
    }
  };
  do_pass(0, 0, std::true_type{});
  if constexpr (KCH <= 8 && !LEAN) {     // (wider inputs stream through the ring once: one pass per workgroup)
    for (int ps = 1; ps < P; ps += 2) {
      do_pass(ps, 1, std::false_type{});
      if (ps + 1 < P) do_pass(ps + 1, 0, std::false_type{});
    }
  }
  // The clamped tail of the weight stream is still in flight: let it land.  Its destination registers
  // must stay the ring's until then (to the compiler an unread asm output is dead at once, and it
  // would hand the registers to the epilogue's values, which the landing data then overwrites):
  // the ties keep the ring alive up to this point.
  wait_vm<0>();
#pragma unroll
  for (int h = 0; h < LOOK; ++h)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) tie(wb[h][nt]);
}


}  // namespace pwp
}  // namespace qasr
