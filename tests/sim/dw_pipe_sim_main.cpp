// CPU replay of the request bookkeeping of the pipelined depthwise kernel (csrc/dw_pipe.hip), in the
// manner of pw_pipe_sim_main.cpp: the kernel function and its planner are compiled for the host
// against pw_pipe_sim_shim.hpp, every lane of every workgroup of a launch runs once to collect the
// wave-wide ballots and once for the record, the records are merged per wave and replayed under
// in-order completion with the latest completion the waits allow.  Checked:
//   * every global address lies inside its operand array, every LDS address inside the launch's
//     dynamic LDS (AddressSanitizer on the build for the plain LDS writes);
//   * the lanes of a wave agree on wait counts, ballots, barriers and stores;
//   * weights and constants (register loads) are complete when they are tied;
//   * the rows of an iteration are complete in LDS when they are read;
//   * nothing is outstanding when a wave ends;
//   * the launch writes every output byte exactly once (rows past the batch, columns past a row and
//     the partner of an odd last tile are rejected by the output resource, not stored).
#include "pw_pipe_sim_shim.hpp"

namespace qasr {
struct Tuning { int dwp_r = 0, dwp_s = 0; };
inline const Tuning& tuning() { static Tuning t; return t; }
}  // namespace qasr

#include "dw_pipe_stripped.hpp"

#include <map>

using namespace qasr;
using sim::merge;
using sim::Wave;

namespace {

struct Case { const char* name; int B, C, T, k, dil, relu, bias, s; };

struct Req { sim::Kind k; int64_t a, b; bool done; };

void replay(const std::vector<sim::Ev>& ev) {
  std::vector<Req> reqs;
  size_t head = 0;
  std::map<int64_t, size_t> reg_req;
  for (const sim::Ev& e : ev) {
    switch (e.k) {
      case sim::ISSUE_LDS: reqs.push_back(Req{e.k, e.a, e.b, false}); break;
      case sim::ISSUE_REG: reg_req[e.a] = reqs.size(); reqs.push_back(Req{e.k, e.a, 0, false}); break;
      case sim::STORE: reqs.push_back(Req{e.k, 0, 0, false}); break;
      case sim::WAIT:
        if (e.b < 0) sim::fail("a run-time wait count is negative");
        while (reqs.size() - head > (size_t)e.a) reqs[head++].done = true;
        break;
      case sim::USE_REG: {
        auto it = reg_req.find(e.a);
        if (it == reg_req.end()) sim::fail("tie of a register no load was issued for");
        if (!reqs[it->second].done) sim::fail("a weight or constant is used before its load has completed");
        break;
      }
      case sim::USE_LDS: {
        // every request of this wave that covers the byte read has to be complete (the latest decides)
        for (long i = (long)reqs.size() - 1; i >= 0; --i)
          if (reqs[i].k == sim::ISSUE_LDS && e.a >= reqs[i].a && e.a < reqs[i].a + reqs[i].b) {
            if (!reqs[i].done) sim::fail("a row in LDS is read before its load has completed");
            break;
          }
        break;
      }
      default: break;
    }
  }
  if (head != reqs.size()) sim::fail("requests are outstanding when the wave ends");
}

template <int KC, int R, int NI>
void run_t(const Case& c, const ConvParams& p, const DwpGeom& g, std::vector<uint8_t>& written) {
  auto& st = sim::S();
  const unsigned gx = 8u * g.c_per_xcd, gy = (unsigned)((p.B + 4 * g.spw - 1) / (4 * g.spw));
  const size_t shmem = (size_t)4 * 3 * R * g.NCH * 16;
  for (unsigned by = 0; by < gy; ++by)
    for (unsigned bx = 0; bx < gx; ++bx) {
      std::vector<unsigned char> lds(shmem, 0);
      st.lds = lds.data(); st.lds_bytes = shmem;
      blockIdx.x = bx; blockIdx.y = by;
      st.where = std::string(c.name) + " workgroup (" + std::to_string(bx) + "," + std::to_string(by) + ")";
      for (int wv = 0; wv < 4; ++wv) {
        Wave w;
        w.lanes.resize(64);
        st.ballots.clear();
        for (int round = 0; round < 2; ++round) {
          st.second_round = round == 1;
          st.count_stores = round == 1;
          for (int l = 0; l < 64; ++l) {
            st.ev.clear(); st.lane = l; st.wave = wv; st.next_uid = 1; st.ballot_idx = 0;
            threadIdx.x = (unsigned)(wv * 64 + l);
            dw_pipe_kernel<KC, R, NI, false>(p, g);
            if (round == 1) w.lanes[l] = st.ev;
          }
        }
        st.lane = -1;
        replay(merge(w));
      }
    }
  (void)written;
}

void run_case(const Case& c) {
  ConvParams p{};
  const int pad = c.dil * (c.k - 1) / 2;
  std::vector<int8_t> x((size_t)c.B * c.C * c.T, 1), y((size_t)c.B * c.C * c.T, 0), w((size_t)c.C * c.k, 1);
  std::vector<int32_t> bias(c.C, 3), m(c.C, 1 << 30), s(c.C, c.s);
  p.x = x.data(); p.w = w.data(); p.bias = c.bias ? bias.data() : nullptr; p.m = m.data(); p.s = s.data(); p.y = y.data();
  p.xbs = (int64_t)c.C * c.T; p.ybs = p.xbs;
  p.B = c.B; p.Cin = c.C; p.Cout = c.C; p.Tin = c.T; p.Tout = c.T;
  p.k = c.k; p.stride = 1; p.dil = c.dil; p.pl = pad; p.depthwise = 1; p.relu = c.relu;
  DwpGeom g{};
  Plan pl{};
  auto& st = sim::S();
  st.where = c.name;
  if (!plan(p, g, pl)) sim::fail("the planner does not take this case");
  st.regions = {{"x", (const unsigned char*)x.data(), x.size(), false}, {"w", (const unsigned char*)w.data(), w.size(), false},
                {"bias", (const unsigned char*)bias.data(), bias.size() * 4, false}, {"m", (const unsigned char*)m.data(), m.size() * 4, false},
                {"s", (const unsigned char*)s.data(), s.size() * 4, false}, {"y", (const unsigned char*)y.data(), y.size(), true}};
  std::vector<uint8_t> written(y.size(), 0);
  st.written = &written;
  st.y_base = (const unsigned char*)y.data();
  bool ran = false;
#define QASR_SIM(K, RR, N) if (pl.KC == K && pl.R == RR && pl.NI == N) { run_t<K, RR, N>(c, p, g, written); ran = true; }
  QASR_SIM(1, 1, 1) QASR_SIM(2, 1, 1) QASR_SIM(1, 2, 1) QASR_SIM(1, 1, 2) QASR_SIM(4, 1, 2)
#undef QASR_SIM
  if (!ran) sim::fail("no instantiation for plan KC " + std::to_string(pl.KC) + " R " + std::to_string(pl.R) + " NI " + std::to_string(pl.NI));
  size_t once = 0;
  for (uint8_t v : written) once += v == 1;
  st.where = c.name;
  if (once != written.size())
    sim::fail("output bytes written exactly once: " + std::to_string(once) + " of " + std::to_string(written.size()));
  std::printf("ok %-44s plan KC %d R %d NI %d S %d, %zu output bytes\n", c.name, pl.KC, pl.R, pl.NI, pl.S, written.size());
}

}  // namespace

int main() {
  const Case cases[] = {
      //  name                                        B   C   T    k  dil relu bias s
      {"k 33, rows of 160 frames", 12, 8, 160, 33, 1, 0, 0, 40},
      {"k 63, rows of 800 frames, batch 32", 32, 3, 800, 63, 1, 1, 0, 38},
      {"k 33, two rows per iteration", 48, 2, 160, 33, 1, 0, 1, 40},
      {"k 33, rows of 1200 frames (two slices)", 12, 2, 1200, 33, 1, 0, 0, 30},
      {"k 87 dilation 2", 12, 2, 800, 87, 2, 0, 0, 40},
      {"k 39, ragged batch 13", 13, 9, 320, 39, 1, 1, 1, 36},
  };
  for (const Case& c : cases) run_case(c);
  std::printf("all cases passed\n");
  return 0;
}
