// Environment overrides of the kernel choices (see tuning.hpp), parsed once.
#include "tuning.hpp"

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <mutex>

namespace qasr {

namespace {

std::mutex g_mu;
Tuning g_tuning;
std::atomic<bool> g_loaded{false};

Tuning read_env() {
  Tuning t;
  t.no_pw_pipe = getenv("QASR_NO_PW_PIPE") != nullptr;
  t.no_conv_pipe = getenv("QASR_NO_CONV_PIPE") != nullptr;
  t.team = getenv("QASR_TEAM") != nullptr;
  t.cp_plain_order = getenv("QASR_CP_PLAIN_ORDER") != nullptr;
  t.no_pw_lean = getenv("QASR_NO_PW_LEAN") != nullptr;
  t.pw_lean_force = getenv("QASR_PW_LEAN") != nullptr;
  t.pw_lean_no_res = getenv("QASR_PW_LEAN_NO_RES") != nullptr;
  t.pwp_nopipe = getenv("QASR_PWP_NOPIPE") != nullptr;
  if (const char* e = getenv("QASR_PWP_MT")) t.pwp_mt = atoi(e);
  if (const char* e = getenv("QASR_PWP_SPLIT")) t.pwp_split = atoi(e);
  if (const char* e = getenv("QASR_DWP")) {
    int r = 0, s = 0;
    if (sscanf(e, "%d,%d", &r, &s) == 2) { t.dwp_r = r; t.dwp_s = s; }
  }
  if (const char* e = getenv("QASR_DW_R")) t.dw_r = atoi(e);
  if (const char* e = getenv("QASR_CP_TILE")) {
    int mt = 0, nt = 0;
    if (sscanf(e, "%d,%d", &mt, &nt) >= 1) { t.cp_mt = mt; t.cp_nt = nt; }
  }
  if (const char* e = getenv("QASR_PWT_MT")) t.pwt_mt = atoi(e);
  if (const char* e = getenv("QASR_SLOT_DEPTH")) {
    const int d = atoi(e);
    if (d >= 0 && d <= 16) t.slot_depth = d;
  }
  return t;
}

}  // namespace

const Tuning& tuning() {
  if (!g_loaded.load(std::memory_order_acquire)) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_loaded.load(std::memory_order_relaxed)) {
      g_tuning = read_env();
      g_loaded.store(true, std::memory_order_release);
    }
  }
  return g_tuning;
}

void tuning_reload() {
  std::lock_guard<std::mutex> lk(g_mu);
  g_tuning = read_env();
  g_loaded.store(true, std::memory_order_release);
}

}  // namespace qasr
