// CPU replay of the request bookkeeping of the pipelined pointwise tile (csrc/pw_pipe_body.hpp).
// The tile function is compiled for the host against pw_pipe_sim_shim.hpp and run once per lane of
// every wave of every workgroup of a launch; the lanes' event lists are merged into the wave's
// instruction stream (a request exists if at least one lane takes part), and the stream is replayed
// under the one property the kernels rely on: a wave's vector-memory requests complete in the
// order they were issued, and `s_waitcnt vmcnt(n)` returns once at most n are outstanding, not
// earlier (the latest completion the hardware may choose).  Checked:
//   * every global address lies inside its operand array, every LDS address inside the
//     workgroup's allocation (the build adds AddressSanitizer for the plain LDS reads and writes);
//   * the lanes of a wave agree on everything that has to be wave-uniform (wait counts, values
//     passed to readfirstlane, barriers, stores);
//   * a register of the weight ring is used (tie) only after its load has completed;
//   * an activation chunk in LDS is read only after this wave's rows of it have completed, and
//     they have completed before the barrier that publishes the chunk to the other waves;
//   * a load into an LDS chunk slot that has been read (the ring of the wide inputs, the residual
//     rows of the lean form) is issued only behind a barrier that every reader has passed;
//   * nothing is outstanding when the tile returns;
//   * the launch writes every output byte exactly once.
#include "pw_pipe_sim_shim.hpp"
#include "pw_pipe_body_stripped.hpp"

#include <deque>
#include <map>

using namespace qasr;
using namespace qasr::pwp;
using sim::Wave;
using sim::merge;

namespace {

struct Case {
  const char* name;
  int MT, KCH, lean;       // instantiation
  int B, T, Cout;          // shape (Cin = 64 KCH)
  int res, relu, bias, splits;
  int slow_pass;           // a pass whose s is below 33 (unpipelined 64-bit epilogue), -1 for none
};

struct Req { sim::Kind k; int64_t a, b; bool done; };

void replay(const std::vector<sim::Ev>& ev, int KCH, size_t xtile_bytes) {
  std::vector<Req> reqs;
  size_t head = 0;                                  // first request that has not completed
  std::map<int64_t, size_t> reg_req;                // uid -> request index
  int barriers = 0;
  std::map<int64_t, int> read_in_step;              // chunk slot -> last chunk step (barriers passed - 1) that read it
  for (const sim::Ev& e : ev) {
    switch (e.k) {
      case sim::ISSUE_LDS:
        // A load into a chunk slot that has been read: every wave reads a chunk in the same step, and a
        // wave that has passed barrier b knows the others are done with step b - 1.
        if ((size_t)e.a < xtile_bytes) {
          auto it = read_in_step.find(e.a / 8192);
          if (it != read_in_step.end() && barriers < it->second + 2)
            sim::fail("a load into an LDS chunk slot is issued while other waves may still be reading the slot");
        }
        reqs.push_back(Req{e.k, e.a, e.b, false});
        break;
      case sim::ISSUE_REG: reg_req[e.a] = reqs.size(); reqs.push_back(Req{e.k, e.a, 0, false}); break;
      case sim::STORE: reqs.push_back(Req{e.k, 0, 0, false}); break;
      case sim::WAIT:
        if (e.k == sim::WAIT && e.b < 0) sim::fail("a run-time wait count is negative: the marks are out of order");
        while (reqs.size() - head > (size_t)e.a) reqs[head++].done = true;
        break;
      case sim::USE_REG: {
        auto it = reg_req.find(e.a);
        if (it == reg_req.end()) sim::fail("tie of a register no load was issued for");
        if (!reqs[it->second].done) sim::fail("a weight register is used before its load has completed");
        break;
      }
      case sim::USE_LDS: {
        if ((size_t)e.a < xtile_bytes) read_in_step[e.a / 8192] = barriers - 1;
        if ((size_t)e.a < xtile_bytes) {            // an activation chunk: this wave's own rows of it
          long r = -1;
          for (long i = (long)reqs.size() - 1; i >= 0 && r < 0; --i)
            if (reqs[i].k == sim::ISSUE_LDS && reqs[i].a / 8192 == e.a / 8192 && (size_t)reqs[i].a < xtile_bytes) r = i;
          if (r >= 0 && !reqs[r].done) sim::fail("an activation chunk is read before this wave's rows of it have completed");
        }
        break;
      }
      case sim::BARRIER: {
        // the barrier of chunk step `barriers` publishes chunk `barriers`: this wave's rows must be in
        const int kc = barriers++;
        if (kc < KCH) {
          long r = -1;
          for (long i = (long)reqs.size() - 1; i >= 0 && r < 0; --i)
            if (reqs[i].k == sim::ISSUE_LDS && (size_t)reqs[i].a < xtile_bytes && reqs[i].a / 8192 == (kc & 7)) r = i;
          if (r >= 0 && !reqs[r].done) sim::fail("a wave passes the barrier of a chunk before its rows of the chunk have completed");
        }
        break;
      }
      case sim::UNIFORM: break;
    }
  }
  if (head != reqs.size()) sim::fail("requests are outstanding when the tile returns");
}

template <int MT, int KCH, bool LEAN>
void run_case(const Case& c) {
  const int Cin = 64 * KCH;
  ConvParams p{};
  std::vector<int8_t> x((size_t)c.B * Cin * c.T, 1), res((size_t)c.B * c.Cout * c.T, 2), y((size_t)c.B * c.Cout * c.T, 0);
  const int co16n = (c.Cout + 15) / 16;
  std::vector<int8_t> w((size_t)co16n * KCH * 1024, 1);
  std::vector<int32_t> bias(c.Cout, 5), m(c.Cout, 1 << 30), s(c.Cout, 40);
  if (c.slow_pass >= 0)
    for (int co = 256 * c.slow_pass; co < std::min(c.Cout, 256 * (c.slow_pass + 1)); ++co) s[co] = 25;
  p.x = x.data(); p.w = w.data(); p.bias = c.bias ? bias.data() : nullptr; p.m = m.data(); p.s = s.data();
  p.res = c.res ? res.data() : nullptr; p.y = y.data();
  p.xbs = (int64_t)Cin * c.T; p.ybs = (int64_t)c.Cout * c.T;
  p.B = c.B; p.Cin = Cin; p.Cout = c.Cout; p.Tin = c.T; p.Tout = c.T;
  p.k = 1; p.stride = 1; p.dil = 1; p.pl = 0; p.depthwise = 0; p.relu = c.relu; p.w_packed = 1;
  PwpGeom g{};
  g.gpr = c.T / 16; g.G = c.B * g.gpr;
  g.passes = (c.Cout + 8 * ROWS - 1) / (8 * ROWS);
  g.co16n = co16n;
  g.tiles = (g.G + MT - 1) / MT;
  g.tiles_per_xcd = (g.tiles + 7) / 8;
  g.splits = LEAN ? g.passes : c.splits;
  g.pps = g.passes / g.splits;
  g.nopipe = LEAN ? 1 : 0;
  const size_t lds_bytes = LEAN ? (size_t)lds_bytes_lean_c<KCH>() : (size_t)lds_bytes_c<KCH>();
  const size_t xtile_bytes = (size_t)(KCH < 8 ? KCH : 8) * 8192;

  auto& st = sim::S();
  st.regions = {{"x", (const unsigned char*)x.data(), x.size(), false}, {"w", (const unsigned char*)w.data(), w.size(), false},
                {"bias", (const unsigned char*)bias.data(), bias.size() * 4, false}, {"m", (const unsigned char*)m.data(), m.size() * 4, false},
                {"s", (const unsigned char*)s.data(), s.size() * 4, false}, {"res", (const unsigned char*)res.data(), res.size(), false},
                {"y", (const unsigned char*)y.data(), y.size(), true}};
  std::vector<uint8_t> written(y.size(), 0);
  st.written = &written;
  st.y_base = (const unsigned char*)y.data();
  const unsigned grid = 8u * g.tiles_per_xcd * g.splits;
  for (unsigned vb = 0; vb < grid; ++vb) {
    std::vector<unsigned char> lds(lds_bytes, 0);            // exactly the launch's dynamic LDS: ASan sees an overrun
    st.lds = lds.data(); st.lds_bytes = lds_bytes;
    Wave waves[8];
    for (int wv = 0; wv < 8; ++wv) {
      waves[wv].lanes.resize(64);
      st.where = std::string(c.name) + " workgroup " + std::to_string(vb);
      // first round: only to learn which constants the wave brings into LDS
      st.dwords.clear();
      st.count_stores = false;
      for (int l = 0; l < 64; ++l) {
        st.ev.clear(); st.lane = l; st.wave = wv; st.next_uid = 1;
        pw_pipe_tile<MT, KCH, false, false, LEAN ? 2 : kLookW, LEAN>(p, g, vb, lds.data(), wv * 64 + l);
      }
      const auto dwords = st.dwords;
      st.count_stores = true;
      for (int l = 0; l < 64; ++l) {
        for (const auto& d : dwords) std::memcpy(lds.data() + d.first, &d.second, 4);
        st.ev.clear(); st.lane = l; st.wave = wv; st.next_uid = 1;
        pw_pipe_tile<MT, KCH, false, false, LEAN ? 2 : kLookW, LEAN>(p, g, vb, lds.data(), wv * 64 + l);
        waves[wv].lanes[l] = st.ev;
      }
    }
    for (int wv = 0; wv < 8; ++wv) {
      st.wave = wv; st.lane = -1;
      replay(merge(waves[wv]), KCH, xtile_bytes);
    }
  }
  size_t once = 0;
  for (uint8_t v : written) once += v == 1;
  if (once != written.size()) {
    st.where = c.name;
    sim::fail("output bytes written " + std::to_string(once) + " of " + std::to_string(written.size()) + " exactly once");
  }
  std::printf("ok %-40s %u workgroups, %zu output bytes\n", c.name, grid, written.size());
}

void dispatch(const Case& c) {
#define QASR_SIM(M, K, L) if (c.MT == M && c.KCH == K && c.lean == L) return run_case<M, K, L>(c);
  QASR_SIM(7, 8, false) QASR_SIM(7, 8, true)
#ifndef SIM_SMALL
  QASR_SIM(7, 4, false) QASR_SIM(4, 8, false) QASR_SIM(5, 4, false)
  QASR_SIM(7, 4, true) QASR_SIM(4, 4, true)
  QASR_SIM(7, 16, false)
#endif
#undef QASR_SIM
  std::fprintf(stderr, "no instantiation for case %s\n", c.name);
  std::exit(4);
}

}  // namespace

int main() {
  const Case cases[] = {
      //  name                          MT KCH lean  B   T   Cout res relu bias splits slow
      {"pipelined 512->512 relu", 7, 8, 0, 2, 208, 512, 0, 1, 1, 1, -1},
      {"pipelined 512->512 residual", 7, 8, 0, 2, 208, 512, 1, 1, 1, 1, -1},
#ifndef SIM_SMALL
      {"pipelined 256->1024 res, pass 1 slow", 7, 4, 0, 1, 160, 1024, 1, 1, 1, 1, 1},
      {"pipelined 512->600 ragged channels", 4, 8, 0, 3, 112, 600, 1, 1, 0, 1, -1},
      {"pipelined 256->768 no relu", 5, 4, 0, 2, 96, 768, 0, 0, 1, 1, -1},
      {"pipelined 512->2048 four workgroups/tile", 7, 8, 0, 1, 128, 2048, 1, 1, 1, 4, -1},
      {"streamed 1024->512 residual", 7, 16, 0, 1, 176, 512, 1, 1, 1, 2, -1},
#endif
      {"lean 512->512", 7, 8, 1, 2, 208, 512, 0, 1, 1, 1, -1},
      {"lean 512->1024 residual", 7, 8, 1, 1, 176, 1024, 1, 1, 1, 1, -1},
#ifndef SIM_SMALL
      {"lean 256->512 residual no relu", 7, 4, 1, 2, 160, 512, 1, 0, 0, 1, -1},
      {"lean 256->256 slow pass", 4, 4, 1, 3, 112, 256, 0, 1, 1, 1, 0},
#endif
  };
  for (const Case& c : cases) dispatch(c);
  std::printf("all cases passed\n");
  return 0;
}
