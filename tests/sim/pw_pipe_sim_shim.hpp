// Host stand-ins for what one tile of the pipelined pointwise kernel (csrc/pw_pipe_body.hpp) asks of
// the GPU, so that the tile function can be compiled for the CPU and run lane by lane: every
// vector-memory request, wait, barrier and use of loaded data is recorded instead of executed, and
// every global address is checked against the operand arrays.  Test infrastructure: nothing of
// the product includes this file.  Values are not simulated (a matrix product returns its
// accumulator): what is checked is the bookkeeping, not the arithmetic, which the GPU parity tests
// cover.
#pragma once
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#define __device__
#define __forceinline__ inline
#define __global__
#define __restrict__
#define __launch_bounds__(...)
#define __shared__ static
#define __align__(n) __attribute__((aligned(n)))
struct SimDim3 { unsigned x = 0, y = 0, z = 0; };
inline SimDim3 threadIdx, blockIdx;

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
using std::max;
using std::min;

namespace sim {

enum Kind { ISSUE_LDS, ISSUE_REG, STORE, WAIT, USE_REG, USE_LDS, BARRIER, UNIFORM };
struct Ev { Kind k; int64_t a, b; };
struct Region { const char* name; const unsigned char* p; size_t n; bool writable; };

struct State {
  std::vector<Ev> ev;                 // of the lane being run
  std::vector<Region> regions;
  std::vector<uint8_t>* written = nullptr;   // per output byte: times stored (whole grid)
  const unsigned char* y_base = nullptr;
  unsigned char* lds = nullptr;
  size_t lds_bytes = 0;
  int lane = 0, wave = 0;
  int next_uid = 1;
  bool count_stores = true;
  std::string where;
  // dword loads into LDS (the per-channel constants) of the whole wave: the lanes run one after the
  // other here, so what the other lanes of the wave load is put in place before each lane runs
  std::vector<std::pair<size_t, uint32_t>> dwords;
  // wave-wide ballots: the first round over a wave's lanes collects them, the second returns them
  std::vector<uint64_t> ballots;
  size_t ballot_idx = 0;
  bool second_round = false;
  std::vector<int32_t> reg_values;       // value behind each register-load tag (index = uid)
};
inline State& S() { static State s; return s; }

[[noreturn]] inline void fail(const std::string& msg) {
  std::fprintf(stderr, "SIM FAILURE (%s, wave %d lane %d): %s\n", S().where.c_str(), S().wave, S().lane, msg.c_str());
  std::exit(3);
}
inline void rec(Kind k, int64_t a = 0, int64_t b = 0) { S().ev.push_back(Ev{k, a, b}); }

inline const Region& region_of(const void* p, size_t n, bool write) {
  const unsigned char* q = (const unsigned char*)p;
  for (const Region& r : S().regions)
    if (q >= r.p && q + n <= r.p + r.n) {
      if (write && !r.writable) fail(std::string("store into read-only operand ") + r.name);
      return r;
    }
  fail("global access outside every operand array");
}
inline size_t lds_off(const void* p, size_t n) {
  const unsigned char* q = (const unsigned char*)p;
  if (q < S().lds || q + n > S().lds + S().lds_bytes) fail("LDS address outside the workgroup's allocation");
  return (size_t)(q - S().lds);
}

// ---- the 64 lane records of a wave, merged into the wave's instruction stream
struct Wave { std::vector<std::vector<Ev>> lanes; };

// (the lanes of a wave read different bytes of the same LDS rows: a use is compared by kind only)
// what only some lanes of a wave may take part in: a load under a lane predicate, and the use of its register
inline bool maskable(Kind k) { return k == ISSUE_LDS || k == ISSUE_REG || k == USE_REG; }
inline bool same(const Ev& a, const Ev& b) { return a.k == b.k && (a.k == USE_LDS || (a.a == b.a && a.b == b.b)); }

// merge the 64 lane streams: events are equal across lanes except that a lane may skip a
// load (masked out) that others issue
inline std::vector<Ev> merge(const Wave& w) {
  std::vector<size_t> pos(64, 0);
  std::vector<Ev> out;
  for (;;) {
    int done = 0;
    for (int l = 0; l < 64; ++l) done += pos[l] == w.lanes[l].size();
    if (done == 64) break;
    // candidate: a masked load that some lane has next, else the common next event
    const Ev* cand = nullptr;
    bool all_equal = true;
    const Ev* first = nullptr;
    for (int l = 0; l < 64; ++l) {
      if (pos[l] == w.lanes[l].size()) { all_equal = false; continue; }
      const Ev& e = w.lanes[l][pos[l]];
      if (!first) first = &e;
      else if (!same(e, *first)) all_equal = false;
    }
    if (all_equal && done == 0) {
      cand = first;
    } else {
      // the earliest-in-program-order differing event is a masked load: pick an ISSUE_LDS some lane has
      for (int l = 0; l < 64 && !cand; ++l)
        if (pos[l] < w.lanes[l].size() && maskable(w.lanes[l][pos[l]].k)) {
          // it must not be the next event of every lane (handled above) and lanes that lack it must be
          // at a later event
          cand = &w.lanes[l][pos[l]];
        }
      if (!cand) {
        std::string d;
        for (int l = 0; l < 64; l += 9)
          if (pos[l] < w.lanes[l].size())
            d += " lane " + std::to_string(l) + ": kind " + std::to_string(w.lanes[l][pos[l]].k) + " a " +
                 std::to_string(w.lanes[l][pos[l]].a) + " b " + std::to_string(w.lanes[l][pos[l]].b) + ";";
        fail("the lanes of a wave disagree on something other than a masked load (event " +
                  std::to_string(out.size()) + ":" + d + ")");
      }
    }
    const Ev c = *cand;
    out.push_back(c);
    int advanced = 0, top = -1;
    for (int l = 0; l < 64; ++l)
      if (pos[l] < w.lanes[l].size() && same(w.lanes[l][pos[l]], c)) { ++pos[l]; ++advanced; top = l; }
    // a load into LDS reaches as far as its highest participating lane (recorded: 64 lanes' worth)
    if (c.k == ISSUE_LDS) out.back().b = c.b / 64 * (top + 1);
    if (!maskable(c.k) && advanced != 64) fail("a wave-uniform event is missing in some lanes");
  }
  return out;
}


}  // namespace sim

// ---- what common.hpp gives the tile (the struct itself is pasted from common.hpp by the test)
#include "conv_params_extract.hpp"

namespace qasr {

inline int32_t mulhi_i32(int32_t a, int32_t b) { return (int32_t)(((int64_t)a * b) >> 32); }
inline int32_t med3_i32(int32_t x, int32_t lo, int32_t hi) { return std::min(std::max(x, lo), hi); }
inline int32_t dyadic_rescale64(int32_t A, int32_t m, int32_t s) {
  long long v = ((long long)A * (long long)m + (1ll << (s - 1))) >> s;
  v = v > (1 << 20) ? (1 << 20) : v;
  v = v < -(1 << 20) ? -(1 << 20) : v;
  return (int32_t)v;
}
template <bool FAST, bool RES>
inline uint32_t requant_pack4(const int32_t (&a)[4], int32_t m, int32_t sh, int32_t rnd, uint32_t resw, int32_t lo,
                              int32_t hi127) {
  uint32_t out = 0;
  for (int i = 0; i < 4; ++i) {
    int32_t v = FAST ? (mulhi_i32(a[i], m) + rnd) >> sh : dyadic_rescale64(a[i], m, sh < 1 ? 1 : sh);
    if (RES) v += (int32_t)(int8_t)(resw >> (8 * i));
    out |= (uint32_t)(uint8_t)med3_i32(v, lo, hi127) << (8 * i);
  }
  return out;
}

// ---- what vmem.hpp gives the tile
inline void direct_load_n(const void* gptr, const unsigned char* lds_wave_base, int n) {
  sim::region_of(gptr, n, false);
  // (the bytes of this lane must be inside the allocation; lanes that stay out of a load write nothing)
  const size_t off = sim::lds_off(lds_wave_base + (size_t)n * sim::S().lane, n) - (size_t)n * sim::S().lane;
  std::memcpy(sim::S().lds + off + (size_t)n * sim::S().lane, gptr, n);      // (data as if it had landed at once)
  if (n == 4) {
    uint32_t v;
    std::memcpy(&v, gptr, 4);
    sim::S().dwords.push_back({off + 4 * (size_t)sim::S().lane, v});
  }
  sim::rec(sim::ISSUE_LDS, (int64_t)off, 64 * n);
}
inline void direct_load16(const void* g, const unsigned char* l) { direct_load_n(g, l, 16); }
inline void direct_load16_dev(const void* g, const unsigned char* l) { direct_load_n(g, l, 16); }
template <bool DEV> inline void direct_load16_scope(const void* g, const unsigned char* l) { direct_load_n(g, l, 16); }
inline void direct_load4(const void* g, const unsigned char* l) { direct_load_n(g, l, 4); }

inline v4i make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t a = (uint64_t)(uintptr_t)base;
  return (v4i){(int)(uint32_t)a, (int)(uint32_t)(a >> 32), (int)bytes, 0};
}
constexpr uint32_t kUidTag = 0x5a000000u;
inline v4i bload16(v4i rsrc, uint32_t voff, uint32_t soff) {
  const unsigned char* base = (const unsigned char*)(uintptr_t)(((uint64_t)(uint32_t)rsrc.y << 32) | (uint32_t)rsrc.x);
  const uint64_t off = (uint64_t)voff + soff;
  if (off + 16 > (uint32_t)rsrc.z) sim::fail("buffer load beyond the resource's size");
  sim::region_of(base + off, 16, false);
  const int uid = sim::S().next_uid++;
  sim::rec(sim::ISSUE_REG, uid);
  return (v4i){(int)(kUidTag | (uint32_t)uid), 0, 0, 0};
}
template <int N> inline void wait_vm() { sim::rec(sim::WAIT, N); }
inline void wait_vm_dyn(int n) {
  sim::rec(sim::UNIFORM, n);
  sim::rec(sim::WAIT, n >= 32 ? 32 : (n < 0 ? 0 : n), n);
}
inline void tie(v4i& v) {
  if (((uint32_t)v.x & 0xff000000u) == kUidTag) {
    sim::rec(sim::USE_REG, (int64_t)((uint32_t)v.x & 0x00ffffffu));
  }
}
// one dword / one sign-extended byte into a register: the tag stands for the value until the tie
inline int32_t reg_load(const void* p, int bytes) {
  sim::region_of(p, bytes, false);
  int32_t v = 0;
  if (bytes == 4) std::memcpy(&v, p, 4);
  else v = *(const int8_t*)p;
  auto& st = sim::S();
  const int uid = st.next_uid++;
  if ((size_t)uid >= st.reg_values.size()) st.reg_values.resize(uid + 1);
  st.reg_values[uid] = v;
  sim::rec(sim::ISSUE_REG, uid);
  return (int32_t)(kUidTag | (uint32_t)uid);
}
inline int32_t gload4(const void* p) { return reg_load(p, 4); }
inline int32_t gload_i8(const void* p) { return reg_load(p, 1); }
inline void tie(int32_t& v) {
  if (((uint32_t)v & 0xff000000u) == kUidTag) {
    const int uid = (int)((uint32_t)v & 0x00ffffffu);
    sim::rec(sim::USE_REG, uid);
    v = sim::S().reg_values[uid];
  }
}

}  // namespace qasr

// ---- compiler builtins the tile uses
struct SimRsrc { unsigned char* p; uint32_t num; };
#define __amdgpu_buffer_rsrc_t SimRsrc
inline SimRsrc sim_make_buffer_rsrc(const void* p, int, int num, int) { return SimRsrc{(unsigned char*)p, (uint32_t)num}; }
#define __builtin_amdgcn_make_buffer_rsrc(p, stride, num, flags) sim_make_buffer_rsrc((const void*)(p), stride, num, flags)
template <typename V>
inline void sim_buffer_store16(V, SimRsrc r, uint32_t off, int, int) {
  sim::rec(sim::STORE);
  if ((uint64_t)off + 16 > r.num) return;                  // rejected by the bounds check, as on the chip
  sim::region_of(r.p + off, 16, true);
  auto& st = sim::S();
  const size_t o = (size_t)(r.p + off - st.y_base);
  if (st.count_stores)
    for (int i = 0; i < 16; ++i) ++(*st.written)[o + i];
}
#define __builtin_amdgcn_raw_buffer_store_b128(v, r, off, soff, aux) sim_buffer_store16(v, r, off, soff, aux)
inline void sim_buffer_store4(uint32_t, SimRsrc r, uint32_t off, int, int) {
  sim::rec(sim::STORE);
  if ((uint64_t)off + 4 > r.num) return;
  sim::region_of(r.p + off, 4, true);
  auto& st = sim::S();
  const size_t o = (size_t)(r.p + off - st.y_base);
  if (st.count_stores)
    for (int i = 0; i < 4; ++i) ++(*st.written)[o + i];
}
#define __builtin_amdgcn_raw_buffer_store_b32(v, r, off, soff, aux) sim_buffer_store4(v, r, off, soff, aux)
inline uint64_t __ballot(bool pred) {
  auto& st = sim::S();
  const size_t i = st.ballot_idx++;
  if (!st.second_round) {
    if (i >= st.ballots.size()) st.ballots.resize(i + 1, 0);
    st.ballots[i] |= (uint64_t)pred << st.lane;
    return (uint64_t)pred << st.lane;
  }
  if (i >= st.ballots.size()) sim::fail("a ballot the first round did not see");
  return st.ballots[i];
}
// a plain 16-byte LDS read of loaded rows (the generator of the depthwise replay routes the one such
// read of that kernel here)
inline v4i sim_lds_read16(const void* p) {
  sim::rec(sim::USE_LDS, (int64_t)sim::lds_off(p, 16));
  return (v4i){0, 0, 0, 0};
}
inline int sim_uniform(int x) { sim::rec(sim::UNIFORM, x); return x; }
inline unsigned sim_uniform(unsigned x) { sim::rec(sim::UNIFORM, (int64_t)x); return x; }
#define __builtin_amdgcn_readfirstlane(x) sim_uniform(x)
#define __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, x, y, z) (c)
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_perm(a, b, c) (0u)
inline void __syncthreads() { sim::rec(sim::BARRIER); }
inline bool __all(bool x) { return x; }
inline v2i sim_lds_tr_read(const void* p) {
  // (recorded per 8 KiB chunk slot: the lanes of a wave read different bytes of the same chunk)
  sim::rec(sim::USE_LDS, (int64_t)(sim::lds_off(p, 8) / 8192 * 8192));
  return (v2i){0, 0};
}
#define __builtin_amdgcn_ds_read_tr8_b64_v2i32(p) sim_lds_tr_read((const void*)(uintptr_t)(p))
