// A run of consecutive encoder layers in ONE kernel launch: persistent workgroups, one per compute
// unit, that walk the layer list with barriers only among the workgroups of one XCD.
//
// Why.  Launched layer by layer, every layer of the batch-32 QuartzNet pays about 5 us before its own
// work starts (the queue's gap between two dependent kernels plus the first memory round trips), as
// much as the work itself.  The utterances of a batch are independent, so nothing of a layer's
// output has to cross from one part of the chip to another: here each XCD (32 compute units around
// one L2) takes its own share of the batch items through the whole run of layers.  A layer boundary
// then needs no more than
//   - every wave waits until its stores are acknowledged (they are in the XCD's L2 then),
//   - a counter in that L2 that the team's workgroups bump and poll               (0.9 us measured),
//   - device-scope loads (sc1) for everything another workgroup wrote: they never hit in the
//     compute unit's vector cache and are served by the L2.  (There is no cheaper way to drop stale
//     vector-cache lines on this chip: `buffer_inv sc0` leaves them in place, `buffer_inv sc1` also
//     empties the L2 and takes 15 us.)
// The activations of a team (4 utterances: 1.6 MB per layer in, as much out) stay in its 4 MB L2 from
// layer to layer.
//
// Teams are formed at run time from the XCC id register, not from an assumed placement: a workgroup
// joins the team of the XCD it really runs on, and the batch is split over the XCDs that turned up.
// All waits are bounded (a poll limit of about a second; the first workgroup to give up raises a flag
// that ends every other wait) and every wave reaches the end of the kernel.  The host refuses shapes
// the layer bodies do not take; those layers run as ordinary launches before and after.
//
// Layer bodies: the pointwise tile of pw_pipe.hip (pw_pipe_body.hpp) and a depthwise body of the same
// arithmetic as dw_pipe.hip (banded-Toeplitz product on the int8 matrix cores) re-cut for a team:
// a wave owns whole channels of the team's utterances, the Toeplitz operand of a channel comes
// ready-made from memory (the weights are static: built once when the encoder is created).
#include "kernels.hpp"
#include "pw_pipe_body.hpp"
#include "team.hpp"
#include "tuning.hpp"
#include "vmem.hpp"

#include <type_traits>

namespace qasr {

namespace {

constexpr unsigned kMaxPolls = 1000000;        // per wait; a poll is a round trip to the L2 or to memory (0.5 - 2 us)
constexpr int kTeamMT = 7;                     // groups per pointwise tile
constexpr int kTeamLook = 2;                   // weight chunks ahead (4 in the stand-alone kernel: 16 registers more than this kernel has)

// The thread's index in the workgroup, rebuilt from the wave's index (kept in LDS like the rest of
// the kernel's state) and the lane's position in the wave, so that the register the hardware hands
// the index over in need not stay reserved through the layer bodies.
// (Computed anew at every use: the empty volatile asm keeps the compiler from computing it once
// ahead of the layer loop and holding it in a register through every layer body.)
__device__ __forceinline__ int lane_id() {
  int l = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  asm volatile("" : "+v"(l));
  return l;
}

__device__ __forceinline__ unsigned load_dev_u32(const unsigned* a) {     // device scope: past the vector cache
  unsigned v;
  asm volatile("global_load_dword %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(a) : "memory");
  return v;
}

// Barrier among the `tsize` workgroups of one team (all on one XCD).  `target` = arrivals that
// complete it (the counter only grows during a launch).  Returns false if a wait was abandoned
// here or elsewhere: the caller leaves the kernel.  Needs every wave's vector-memory requests to
// have completed before the count (the waves wait themselves: vmcnt is per wave).
__device__ __forceinline__ bool team_barrier(TeamCtl* c, unsigned xcc, unsigned target, unsigned* lds_flag, bool first_thread) {
  wait_vm<0>();                                   // this wave's stores are in the L2
  __syncthreads();
  if (first_thread) {
    unsigned* cnt = &c->team_count[xcc * 32];
    const unsigned one = 1;
    asm volatile("global_atomic_add %0, %1, off" :: "v"(cnt), "v"(one) : "memory");
    unsigned polls = 0, ok = 1;
    while (load_dev_u32(cnt) < target) {
      if (++polls > kMaxPolls || ((polls & 127) == 0 && load_dev_u32(&c->abort))) {
        __hip_atomic_store(&c->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    *lds_flag = ok;
  }
  __syncthreads();
  return *lds_flag != 0;
}

// ---------------------------------------------------------------------------------------------
// Depthwise layer of a team.  Arithmetic as in dw_pipe.hip:
//     Y[m, n] = sum_kappa A[m, kappa] * X[kappa, n]             (v_mfma_i32_16x16x64_i8)
//     column n = one 16-frame group, m = frame in the group; X[kappa, n] = x[16 n - PH*16 + kappa]
//     A[m, kappa] = w[j] where kappa - m - delta == j * dilation  (ready-made: TeamOp::w)
// Wave `tw` of the team's `tws` waves owns channels tw, tw + tws, ...; an iteration is one channel
// and up to R of the team's utterances, whose 16-frame groups form one flat list of columns cut into
// tiles of 16.  Everything an iteration needs is requested two iterations ahead by direct
// global->LDS loads into one of three per-wave buffers (nothing in flight lives in a register):
//     [R rows][NCH chunks of 16 B] | Toeplitz operand, KC x 1 KiB in register layout | m, s, bias
// always KC + 1 + R requests; an iteration ends with one store per tile, always issued (rejected by
// its offset where the tile runs past the rows), so the counts a wave waits with are fixed.
struct DwTeam {
  const int8_t* x;          // first utterance of the team, channel 0
  int8_t* y;
  const int8_t* toep;       // [C][KC][64 lanes][16 B]
  const int32_t *bias, *m, *s;
  int64_t xbs, ybs;
  int32_t Bt, C, T, G, NCH, PH, relu;
};

template <int KC, int R>
constexpr int dw_team_wave_bytes(int NCH) { return 3 * (R * NCH * 16 + KC * 1024 + 64); }

template <int KC, int R>
__device__ __forceinline__ void dw_team(const DwTeam& d, unsigned tw, unsigned tws, unsigned char* lds, int wave) {
  const int lane = lane_id();          // (what derives from the lane stays inside the layer: see pw_pipe_body.hpp)
  const int n = lane & 15, gi = lane >> 4;
  const int rowbytes = d.NCH * 16;
  const int bufbytes = R * rowbytes + KC * 1024 + 64;
  unsigned char* const my = lds + (size_t)wave * 3 * bufbytes;

  const int rg = (d.Bt + R - 1) / R;                                   // row groups per channel
  const int n_ch = (int)tw < d.C ? (d.C - (int)tw + (int)tws - 1) / (int)tws : 0;
  const int n_it = __builtin_amdgcn_readfirstlane(n_ch * rg);
  if (n_it == 0) return;                                               // whole wave

  // chunk u of a row holds frames 16 (u - PH) .. +15; chunks outside the row are zeros, written
  // once here; their lanes stay out of every load
  const int tchunk = 16 * (lane - d.PH);
  const bool lane_in = lane < d.NCH && tchunk >= 0 && tchunk < d.T;
  if (lane < d.NCH && !lane_in)
    for (int q = 0; q < 3; ++q)
      for (int r = 0; r < R; ++r)
        *reinterpret_cast<v4i*>(my + q * bufbytes + r * rowbytes + lane * 16) = (v4i){0, 0, 0, 0};

  auto issue = [&](int it, int buf) __attribute__((always_inline)) {
    const int ci = it / rg, row0 = (it - ci * rg) * R;
    const int c = (int)tw + ci * (int)tws;
    unsigned char* const b = my + buf * bufbytes;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc)
      direct_load16(d.toep + (((int64_t)c * KC + kc) * 64 + lane) * 16, b + R * rowbytes + kc * 1024);
    {                                                                  // lanes 0..2: m, s, bias (m again if there is none)
      const int32_t* cp = lane == 0 ? d.m + c : lane == 1 ? d.s + c : (d.bias ? d.bias + c : d.m + c);
      if (lane < 3) direct_load4(cp, b + R * rowbytes + KC * 1024);
    }
    const int8_t* xc = d.x + (int64_t)c * d.T + tchunk;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = min(row0 + r, d.Bt - 1);                          // past the end: the last row again
      if (lane_in) direct_load16_dev(xc + (int64_t)row * d.xbs, b + r * rowbytes);
    }
  };
  constexpr int cI = KC + 1 + R;
  const int NTI = (R * d.G + 15) / 16;                                   // tiles (= stores) per iteration
  const int cS = NTI;
  const int lo = d.relu ? 0 : -128;
  const int32_t hi127 = 127;

  auto iteration = [&](int it, int buf) __attribute__((always_inline)) {
    const int ci = it / rg, row0 = (it - ci * rg) * R;
    const int c = (int)tw + ci * (int)tws;
    // everything up to this iteration's own requests has to be complete: only the requests of the
    // next two iterations and the stores of the last two may still be under way
    wait_vm_dyn((it + 1 < n_it ? cI : 0) + (it + 2 < n_it ? cI : 0) + (it >= 1 ? cS : 0) + (it >= 2 ? cS : 0));
    asm volatile("" ::: "memory");
    const unsigned char* const rows_lds = my + buf * bufbytes;
    const unsigned char* const a_lds = rows_lds + R * rowbytes;
    const int32_t* const c_lds = reinterpret_cast<const int32_t*>(a_lds + KC * 1024);
    v4i a[KC];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) a[kc] = *reinterpret_cast<const v4i*>(a_lds + kc * 1024 + lane * 16);
    const int32_t m_u = __builtin_amdgcn_readfirstlane(c_lds[0]);      // one channel per wave: uniform
    const int32_t s_u = __builtin_amdgcn_readfirstlane(c_lds[1]);
    const int32_t b_u = d.bias ? __builtin_amdgcn_readfirstlane(c_lds[2]) : 0;
    const int Rv = min(R, d.Bt - row0);
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(
        d.y + (int64_t)row0 * d.ybs + (int64_t)c * d.T, 0,
        (int)((uint32_t)(Rv - 1) * (uint32_t)d.ybs + (uint32_t)d.T), 0x00027000);
    const bool fast = s_u >= 33;
    const int sh = fast ? s_u - 32 : s_u, rnd = fast ? 1 << ((s_u - 33) & 31) : 0;
    const v4i bias4 = {b_u, b_u, b_u, b_u};
    auto tiles = [&](auto fast_tag) __attribute__((always_inline)) {
      constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll 2
      for (int j = 0; j < NTI; ++j) {
        int col = 16 * j + n, rr = 0;
#pragma unroll
        for (int q = 1; q < R; ++q)
          if (col >= q * d.G) rr = q;
        int grp = col - rr * d.G;
        const bool in = grp < d.G;                                       // (else rr == R - 1 and the column is past the rows)
        if (!in) grp = 0;                                                // reads stay inside the buffer
        const unsigned char* src = rows_lds + (((rr * d.NCH) + grp + gi) << 4);
        v4i acc = bias4;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
          const v4i xb = *reinterpret_cast<const v4i*>(src + kc * 64);
          acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[kc], xb, acc, 0, 0, 0);
        }
        const int32_t a4[4] = {acc[0], acc[1], acc[2], acc[3]};
        const uint32_t pk = requant_pack4<FAST, false>(a4, m_u, sh, rnd, 0u, lo, hi127);
        const uint32_t off = in ? (uint32_t)rr * (uint32_t)d.ybs + (uint32_t)(16 * grp + 4 * gi) : 0xfffffff0u;
        __builtin_amdgcn_raw_buffer_store_b32(pk, yrs, off, 0, 0);
      }
    };
    if (fast) tiles(std::true_type{}); else tiles(std::false_type{});
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // every LDS read of this buffer has returned
    if (it + 3 < n_it) issue(it + 3, buf);
  };

  issue(0, 0);
  if (1 < n_it) issue(1, 1);
  if (2 < n_it) issue(2, 2);
  for (int it0 = 0; it0 < n_it; it0 += 3) {
#pragma unroll
    for (int h = 0; h < 3; ++h) {
      if (it0 + h >= n_it) break;
      iteration(it0 + h, h);
    }
  }
  wait_vm<0>();
}

// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ const int8_t* slot_ptr(int kind, int64_t off, const int8_t* x, const int8_t* ws, const int8_t* y) {
  return (kind == 0 ? x : kind == 1 ? ws : y) + off;
}

// Everything that lives as long as the kernel is parked in LDS and read again where it is needed:
// the layer bodies need nearly every scalar and vector register there is (kept in registers across
// them, this state made the compiler spill, and a spill is a vector-memory request nobody counted).
struct TeamState {
  unsigned long long ops, x, ws, y, ctl;     // the kernel's pointer arguments
  unsigned n_ops, B, stamps_on;
  unsigned xcc, slot, n_teams, team, tsize;  // this workgroup's place
  unsigned item0, Bt;                        // the team's utterances
  unsigned ok, barriers, flag;               // formation succeeded; barriers passed so far; barrier result
};

__device__ __forceinline__ unsigned uni(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ unsigned long long uni64(unsigned long long v) {
  return ((unsigned long long)uni((unsigned)(v >> 32)) << 32) | uni((unsigned)v);
}

// The layer record with every field in scalar registers (the loads below are ordinary loads; whatever
// registers they arrive in, the copies are wave-uniform by construction, which the hand-written loads
// of the layer bodies need for their resource descriptors and base addresses).
__device__ __forceinline__ TeamOp load_op(const TeamOp* src) {
  TeamOp o;
  o.kind = (int)uni((unsigned)src->kind); o.sync_before = (int)uni((unsigned)src->sync_before);
  o.in_kind = (int)uni((unsigned)src->in_kind); o.res_kind = (int)uni((unsigned)src->res_kind);
  o.out_kind = (int)uni((unsigned)src->out_kind); o.variant = (int)uni((unsigned)src->variant);
  o.in_off = (int64_t)uni64((unsigned long long)src->in_off); o.res_off = (int64_t)uni64((unsigned long long)src->res_off);
  o.out_off = (int64_t)uni64((unsigned long long)src->out_off);
  o.xbs = (int64_t)uni64((unsigned long long)src->xbs); o.ybs = (int64_t)uni64((unsigned long long)src->ybs);
  o.Cin = (int)uni((unsigned)src->Cin); o.Cout = (int)uni((unsigned)src->Cout); o.T = (int)uni((unsigned)src->T);
  o.relu = (int)uni((unsigned)src->relu);
  o.w = reinterpret_cast<const int8_t*>(uni64((unsigned long long)(uintptr_t)src->w));
  o.bias = reinterpret_cast<const int32_t*>(uni64((unsigned long long)(uintptr_t)src->bias));
  o.m = reinterpret_cast<const int32_t*>(uni64((unsigned long long)(uintptr_t)src->m));
  o.s = reinterpret_cast<const int32_t*>(uni64((unsigned long long)(uintptr_t)src->s));
  o.delta = (int)uni((unsigned)src->delta); o.PH = (int)uni((unsigned)src->PH); o.NCH = (int)uni((unsigned)src->NCH);
  o.G = (int)uni((unsigned)src->G); o.KC = (int)uni((unsigned)src->KC); o.pad_ = 0;
  return o;
}

// What a layer needs from the layer record and the kernel's state, gathered anew wherever it is used
// (so that none of it has to survive a layer body in registers).
struct LayerView {
  TeamOp op;
  const int8_t* xin;
  const int8_t* res;
  int8_t* yout;
  unsigned slot, tsize;
  int Bt;
};
__device__ __forceinline__ LayerView view_layer(int i, const volatile TeamState* st) {
  LayerView v;
  v.op = load_op(reinterpret_cast<const TeamOp*>(uni64(st->ops)) + i);
  v.slot = uni(st->slot);
  v.tsize = uni(st->tsize);
  v.Bt = (int)uni(st->Bt);
  const int item0 = (int)uni(st->item0);
  const int8_t* const x = reinterpret_cast<const int8_t*>(uni64(st->x));
  const int8_t* const ws = reinterpret_cast<const int8_t*>(uni64(st->ws));
  const int8_t* const y = reinterpret_cast<const int8_t*>(uni64(st->y));
  v.xin = slot_ptr(v.op.in_kind, v.op.in_off, x, ws, y) + (int64_t)item0 * v.op.xbs;
  v.yout = const_cast<int8_t*>(slot_ptr(v.op.out_kind, v.op.out_off, x, ws, y)) + (int64_t)item0 * v.op.ybs;
  v.res = v.op.res_kind < 0 ? nullptr : slot_ptr(v.op.res_kind, v.op.res_off, x, ws, y) + (int64_t)item0 * v.op.ybs;
  return v;
}

// pointwise layer: the team's tiles round-robin over its workgroups
template <int KCH>
__device__ __forceinline__ void team_pointwise(int i, const volatile TeamState* st, unsigned char* lds, int wave) {
  for (unsigned vb = uni(st->slot);; vb += uni(st->tsize)) {
    const LayerView v = view_layer(i, st);       // (per tile: nothing of it stays live across the tile)
    ConvParams p{};
    p.x = v.xin; p.w = v.op.w; p.bias = v.op.bias; p.m = v.op.m; p.s = v.op.s; p.y = v.yout; p.res = v.res;
    p.xbs = v.op.xbs; p.ybs = v.op.ybs;
    p.B = v.Bt; p.Cin = v.op.Cin; p.Cout = v.op.Cout; p.Tin = v.op.T; p.Tout = v.op.T;
    p.k = 1; p.stride = 1; p.dil = 1; p.pl = 0; p.depthwise = 0; p.relu = v.op.relu; p.w_packed = 1;
    pwp::PwpGeom g;
    g.gpr = v.op.T / 16;
    g.G = v.Bt * g.gpr;
    g.passes = (v.op.Cout + 8 * pwp::ROWS - 1) / (8 * pwp::ROWS);
    g.co16n = (v.op.Cout + 15) / 16;
    g.tiles = (g.G + kTeamMT - 1) / kTeamMT;
    g.tiles_per_xcd = g.tiles;
    g.splits = 1;
    g.pps = g.passes;
    g.nopipe = 0;
    if (vb >= (unsigned)g.tiles) break;
    pwp::pw_pipe_tile<kTeamMT, KCH, false, true, kTeamLook>(p, g, vb, lds, wave * 64 + lane_id());
    __syncthreads();                              // the tile in LDS is free again
  }
}

template <int KC, int R>
__device__ __forceinline__ void team_depthwise(int i, const volatile TeamState* st, unsigned char* lds, int wave) {
  const LayerView v = view_layer(i, st);
  DwTeam d;
  d.x = v.xin; d.y = v.yout; d.toep = v.op.w; d.bias = v.op.bias; d.m = v.op.m; d.s = v.op.s;
  d.xbs = v.op.xbs; d.ybs = v.op.ybs; d.Bt = v.Bt; d.C = v.op.Cout; d.T = v.op.T; d.G = v.op.G; d.NCH = v.op.NCH;
  d.PH = v.op.PH; d.relu = v.op.relu;
  dw_team<KC, R>(d, v.slot * 8 + (unsigned)wave, v.tsize * 8, lds, wave);
}

__device__ __forceinline__ void team_layer(int i, const volatile TeamState* st, unsigned char* lds, int wave) {
  const TeamOp* rec = reinterpret_cast<const TeamOp*>(uni64(st->ops)) + i;
  const int kind = (int)uni((unsigned)rec->kind), variant = (int)uni((unsigned)rec->variant);
  if (kind == 0) {
    if (variant == 4) team_pointwise<4>(i, st, lds, wave);
    else team_pointwise<8>(i, st, lds, wave);
  } else {
    if (variant == 1) team_depthwise<1, 4>(i, st, lds, wave);
    else if (variant == 2) team_depthwise<2, 4>(i, st, lds, wave);
    else team_depthwise<3, 3>(i, st, lds, wave);
  }
}

__global__ __launch_bounds__(512) void team_kernel(const TeamOp* __restrict__ ops, int n_ops, const int8_t* x,
                                                    int8_t* ws, int8_t* y, int B, TeamCtl* ctl, int stamps_on) {
  extern __shared__ __align__(128) unsigned char lds[];
  __shared__ TeamState st_;
  volatile TeamState& st = st_;     // every read is a read of LDS: nothing of it is carried in registers

  // ---- join the team of the XCD this workgroup runs on; wait until every workgroup has joined
  if (threadIdx.x == 0) {
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    xcc &= 15u;
    const unsigned slot = __hip_atomic_fetch_add(&ctl->team_n[xcc], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_fetch_add(&ctl->registered, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned polls = 0, ok = 1;
    while (load_dev_u32(&ctl->registered) < gridDim.x) {
      if (++polls > kMaxPolls || ((polls & 127) == 0 && load_dev_u32(&ctl->abort))) {
        __hip_atomic_store(&ctl->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(2);
    }
    // teams = the XCC ids that have members, in ascending order
    unsigned n_teams = 0, my_team = 0, my_size = 0;
    if (ok) {
      for (unsigned t = 0; t < 16; ++t) {
        const unsigned cnt = load_dev_u32(&ctl->team_n[t]);
        if (t == xcc) { my_team = n_teams; my_size = cnt; }
        if (cnt) ++n_teams;
      }
    }
    st.ops = (unsigned long long)(uintptr_t)ops; st.x = (unsigned long long)(uintptr_t)x;
    st.ws = (unsigned long long)(uintptr_t)ws; st.y = (unsigned long long)(uintptr_t)y;
    st.ctl = (unsigned long long)(uintptr_t)ctl;
    st.n_ops = (unsigned)n_ops; st.B = (unsigned)B; st.stamps_on = (unsigned)stamps_on;
    st.xcc = xcc; st.slot = slot; st.n_teams = n_teams; st.team = my_team; st.tsize = my_size;
    // the team's utterances (more XCDs than utterances: some teams have nothing to do; nobody waits for them)
    const unsigned ipt = n_teams ? ((unsigned)B + n_teams - 1) / n_teams : 0;
    const unsigned item0 = my_team * ipt;
    st.item0 = item0;
    st.Bt = item0 < (unsigned)B ? min(ipt, (unsigned)B - item0) : 0u;
    st.ok = ok && n_teams && my_size;
    st.barriers = 0;
    st.flag = 1;
  }
  __syncthreads();
  if (!uni(st.ok) || uni(st.Bt) == 0) return;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // the one value kept in a register throughout
  if (uni(st.stamps_on) && uni(st.team) == 0 && uni(st.slot) == 0 && wave == 0 && lane_id() == 0)
    reinterpret_cast<TeamCtl*>(uni64(st.ctl))->stamp[0] = wall_clock64();

  for (int i = 0; i < (int)uni(st.n_ops); ++i) {
    {
      const int sync_before = (int)uni((unsigned)reinterpret_cast<const TeamOp*>(uni64(st.ops))[i].sync_before);
      if (sync_before) {
        TeamCtl* c = reinterpret_cast<TeamCtl*>(uni64(st.ctl));
        const unsigned target = (uni(st.barriers) + 1) * uni(st.tsize);
        const bool first = wave == 0 && lane_id() == 0;
        const bool ok = team_barrier(c, uni(st.xcc), target, &st_.flag, first);
        if (first) st.barriers += 1;                // (read again only after the next __syncthreads)
        if (!ok) return;
      }
    }
    team_layer(i, &st, lds, wave);
    __syncthreads();                                // LDS changes hands between layers
    if (uni(st.stamps_on) && uni(st.team) == 0 && uni(st.slot) == 0 && wave == 0 && lane_id() == 0 && i + 1 < kTeamMaxStamps)
      reinterpret_cast<TeamCtl*>(uni64(st.ctl))->stamp[i + 1] = wall_clock64();
  }
  wait_vm<0>();
}

// one byte per thread: image byte e of lane (m, gi) of chunk kc of channel c = A[m, 64 kc + 16 gi + e]
__global__ void toeplitz_image_kernel(const int8_t* __restrict__ w, int C, int k, int dil, int delta, int KC,
                                      int8_t* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)C * KC * 1024;
  if (idx >= total) return;
  const int e = (int)(idx & 15), lane = (int)((idx >> 4) & 63);
  const int kc = (int)((idx >> 10) % KC), c = (int)((idx >> 10) / KC);
  const int m = lane & 15, gi = lane >> 4;
  const int kap = 64 * kc + 16 * gi + e;
  const int dlt = kap - m - delta;
  int8_t v = 0;
  if (dlt >= 0 && dlt % dil == 0 && dlt / dil < k) v = w[(int64_t)c * k + dlt / dil];
  out[idx] = v;
}

__global__ void team_ctl_clear_kernel(TeamCtl* c) {
  unsigned* p = reinterpret_cast<unsigned*>(c);
  constexpr unsigned n = (unsigned)(offsetof(TeamCtl, stamp) / 4);
  for (unsigned i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0u;
}

constexpr size_t team_lds_bytes() { return (size_t)pwp::lds_bytes_c<8>(); }
// the depthwise buffers of 8 waves fit in that at the largest row the host admits (64 chunks)
static_assert(8 * dw_team_wave_bytes<1, 4>(64) <= (int)team_lds_bytes(), "depthwise KC = 1");
static_assert(8 * dw_team_wave_bytes<2, 4>(64) <= (int)team_lds_bytes(), "depthwise KC = 2");
static_assert(8 * dw_team_wave_bytes<3, 3>(64) <= (int)team_lds_bytes(), "depthwise KC = 3");

}  // namespace

bool team_dw_geometry(const ConvParams& p, TeamOp& t) {
  if (!p.depthwise || p.stride != 1 || p.res || p.act_lut || p.n_res_more) return false;
  if (p.Tin != p.Tout || p.Tin % 16 != 0 || p.xbs % 16 != 0 || p.ybs % 16 != 0) return false;
  if (p.ybs >= 0x10000000LL) return false;                     // 32-bit offsets of up to 4 rows
  const int delta = ((-p.pl) % 16 + 16) % 16;
  const int64_t need = 16 + delta + (int64_t)p.dil * (p.k - 1);
  const int KC = (int)((need + 63) / 64);
  if (KC < 1 || KC > 3) return false;
  const int G = p.Tout / 16;
  const int NCH = G + 4 * KC - 1;
  if (NCH > 64) return false;                                  // one 64-lane request per row
  t.delta = delta;
  t.PH = (p.pl + delta) / 16;
  t.NCH = NCH;
  t.G = G;
  t.KC = KC;
  t.variant = KC;
  return true;
}

bool team_pw_geometry(const ConvParams& p, TeamOp& t) {
  if (!pw_pipe_supported(p) || p.act_lut || p.n_res_more) return false;
  if (p.Cin != 256 && p.Cin != 512) return false;             // the tile stays resident in LDS
  t.variant = p.Cin / 64;
  return true;
}

size_t team_toeplitz_bytes(const TeamOp& t, int C) { return (size_t)C * t.KC * 1024; }

hipError_t launch_toeplitz_image(const int8_t* w, int C, int k, int dil, const TeamOp& t, int8_t* out, hipStream_t st) {
  const int64_t total = (int64_t)C * t.KC * 1024;
  return launch_kernel(toeplitz_image_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w, C, k, dil,
                       t.delta, t.KC, out);
}

hipError_t launch_team(const TeamOp* ops_dev, int n_ops, const int8_t* x, int8_t* ws, int8_t* y, int B, TeamCtl* ctl,
                       int n_workgroups, int stamps_on, hipStream_t st) {
  static std::atomic<uint64_t> lds_raised{0};
  if (const hipError_t e = ensure_max_dynamic_lds((const void*)team_kernel, lds_raised, (int)team_lds_bytes()); e != hipSuccess) return e;
  // the control block is cleared by a kernel (not a memset node: this call may be under graph capture)
  if (const hipError_t e = launch_kernel(team_ctl_clear_kernel, dim3(1), dim3(256), 0, st, ctl); e != hipSuccess)
    return e;
  return launch_kernel(team_kernel, dim3((unsigned)n_workgroups), dim3(512), team_lds_bytes(), st, ops_dev, n_ops, x, ws, y,
                       B, ctl, stamps_on);
}

int team_workgroups() {
  int dev = 0, cus = 0, lds_max = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8) return 0;
  // One workgroup per compute unit: 8 waves of at most 256 registers (two per SIMD) and less LDS
  // than a unit has, so each of them fits, and more than half a unit's LDS, so no unit takes two.
  // All of them are resident together, which the barriers rely on.
  if (hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return 0;
  if ((size_t)lds_max < team_lds_bytes() + 256) return 0;      // (dynamic + the kernel's few static bytes)
  static std::atomic<uint64_t> lds_raised{0};
  const hipError_t ae = ensure_max_dynamic_lds((const void*)team_kernel, lds_raised, (int)team_lds_bytes());
  if (ae != hipSuccess) {
    (void)hipGetLastError();                      // optional path: leave no stale error behind
    return 0;
  }
  return cus;
}

}  // namespace qasr
