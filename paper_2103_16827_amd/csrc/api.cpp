// C ABI of the library: argument validation (before any HIP call), kernel dispatch, and the
// encoder executor (a flat op list over activation slots).  See include/qasr.h.
#include "../../include/qasr.h"
#include "kernels.hpp"
#include "team.hpp"
#include "tuning.hpp"

#include <cmath>
#include <mutex>
#include <new>
#include <vector>

using qasr::ConvParams;

namespace {

thread_local hipError_t g_last_hip = hipSuccess;   // detail behind the last QASR_ERR_HIP

qasr_status hip_status(hipError_t e) {
  if (e == hipSuccess) return QASR_OK;
  g_last_hip = e;
  return QASR_ERR_HIP;
}

constexpr uint32_t kKnownFlags = QASR_FLAG_RELU | QASR_FLAG_W_PACKED;

// Weights have a packed form only for groups == 1 with Cin a multiple of 64 (the matrix-core
// kernels' operand order); otherwise "packed" is the plain order.
bool has_packed_form(const qasr_conv1d_desc* d) { return d->groups == 1 && d->Cin % 64 == 0; }

size_t packed_bytes_of(const qasr_conv1d_desc* d) {
  if (!has_packed_form(d)) return (size_t)((int64_t)d->Cout * (d->groups != 1 ? 1 : d->Cin) * d->k);
  return (size_t)((int64_t)d->k * ((d->Cout + 15) / 16) * 16 * d->Cin);
}

int64_t out_len64(const qasr_conv1d_desc* d) {
  const int64_t span = (int64_t)d->Tin + d->pad_left + d->pad_right - (int64_t)d->dilation * (d->k - 1) - 1;
  return span < 0 ? 0 : span / d->stride + 1;
}

qasr_status check_desc(const qasr_conv1d_desc* d) {
  if (!d) return QASR_ERR_NULL;
  if (d->B < 1 || d->Cin < 1 || d->Cout < 1 || d->Tin < 1 || d->k < 1 || d->stride < 1 ||
      d->dilation < 1 || d->pad_left < 0 || d->pad_right < 0)
    return QASR_ERR_SHAPE;
  if (d->flags & ~kKnownFlags) return QASR_ERR_PARAM;
  if (d->groups != 1 && !(d->groups == d->Cin && d->Cin == d->Cout)) return QASR_ERR_UNSUPPORTED;
  const int64_t Tout = out_len64(d);
  if (Tout < 1 || Tout > 0x7fffffffLL) return QASR_ERR_SHAPE;
  if (d->x_batch_stride < 0 || d->y_batch_stride < 0) return QASR_ERR_SHAPE;
  if (d->x_batch_stride && d->x_batch_stride < (int64_t)d->Cin * d->Tin) return QASR_ERR_SHAPE;
  if (d->y_batch_stride && d->y_batch_stride < (int64_t)d->Cout * Tout) return QASR_ERR_SHAPE;
  return QASR_OK;
}

bool overlaps(const void* a, int64_t na, const void* b, int64_t nb) {
  const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + (uint64_t)nb && b0 < a0 + (uint64_t)na;
}

ConvParams make_params(const qasr_conv1d_desc* d, const int8_t* x, const int8_t* w, const int32_t* bias,
                       const int32_t* m, const int32_t* s, const int8_t* res, int8_t* y) {
  ConvParams p{};
  p.x = x; p.w = w; p.bias = bias; p.m = m; p.s = s; p.res = res; p.y = y;
  p.B = d->B; p.Cin = d->Cin; p.Cout = d->Cout; p.Tin = d->Tin; p.Tout = (int32_t)out_len64(d);
  p.k = d->k; p.stride = d->stride; p.dil = d->dilation; p.pl = d->pad_left;
  p.depthwise = d->groups != 1;
  p.relu = (d->flags & QASR_FLAG_RELU) ? 1 : 0;
  p.w_packed = (has_packed_form(d) && (d->flags & QASR_FLAG_W_PACKED)) ? 1 : 0;
  p.xbs = d->x_batch_stride ? d->x_batch_stride : (int64_t)d->Cin * d->Tin;
  p.ybs = d->y_batch_stride ? d->y_batch_stride : (int64_t)d->Cout * p.Tout;
  return p;
}

enum class Kernel { Generic, DwMfma, DwPipe, GemmMfma, PwTile, PwPipe, ConvPipe };

Kernel pick_kernel(const ConvParams& p) {
  if (p.n_res_more > 0)      // dense-residual layers: the two kernels whose epilogue adds several operands
    return (!p.depthwise && qasr::conv_pipe_supported(p)) ? Kernel::ConvPipe : Kernel::Generic;
  if (p.depthwise) {
    if (qasr::dw_pipe_supported(p)) return Kernel::DwPipe;
    return qasr::dw_mfma_supported(p) ? Kernel::DwMfma : Kernel::Generic;
  }
  if (qasr::pw_pipe_supported(p)) return Kernel::PwPipe;
  if (qasr::pw_tile_supported(p)) return Kernel::PwTile;
  if (qasr::conv_pipe_supported(p)) return Kernel::ConvPipe;
  if (qasr::gemm_mfma_supported(p)) return Kernel::GemmMfma;
  return Kernel::Generic;
}

// kernels whose epilogue applies a unary activation's table (ConvParams::act_lut)
bool applies_act_table(Kernel k) { return k == Kernel::PwPipe || k == Kernel::DwPipe; }

const char* kernel_name(Kernel k) {
  switch (k) {
    case Kernel::DwMfma: return "dw_mfma";
    case Kernel::DwPipe: return "dw_pipe";
    case Kernel::GemmMfma: return "gemm_mfma";
    case Kernel::PwTile: return "pw_tile";
    case Kernel::PwPipe: return "pw_pipe";
    case Kernel::ConvPipe: return "conv_pipe";
    default: return "conv_generic";
  }
}

qasr_status launch_with(Kernel k, const ConvParams& p, hipStream_t st) {
  hipError_t e;
  switch (k) {
    case Kernel::DwMfma: e = qasr::launch_dw_mfma(p, st); break;
    case Kernel::DwPipe: e = qasr::launch_dw_pipe(p, st); break;
    case Kernel::GemmMfma: e = qasr::launch_gemm_mfma(p, st); break;
    case Kernel::PwTile: e = qasr::launch_pw_tile(p, st); break;
    case Kernel::PwPipe: e = qasr::launch_pw_pipe(p, st); break;
    case Kernel::ConvPipe: e = qasr::launch_conv_pipe(p, st); break;
    default: e = qasr::launch_conv_generic(p, st); break;
  }
  return hip_status(e);
}

qasr_status launch(const ConvParams& p, hipStream_t st) { return launch_with(pick_kernel(p), p, st); }

size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

struct qasr_encoder {
  struct Op {
    qasr_conv1d_desc d;
    ConvParams p;          // pointers to weights/constants filled in; x / res / y set per forward
    int32_t in_slot, res_slot, out_slot;
    Kernel kernel;
    int32_t n_more_res = 0;
    int32_t more_res_slots[QASR_MAX_RESIDUALS - 1];
    bool has_act = false;
    bool act_fused = false;   // the layer's own kernel applies it (p.act_lut)
    qasr::ActParams act;   // applied in place to the output when has_act
  };
  std::vector<Op> ops;
  std::vector<size_t> slot_off;   // byte offset of slot i in the workspace (slot 0 unused)
  size_t ws_bytes = 0;
  size_t in_elems = 0, out_elems = 0;   // int8 elements of the network input and output
  int8_t* packed = nullptr;       // device: packed weights of all groups == 1 layers
  // Runs of consecutive ops that one launch of the persistent team kernel executes (team.hip); the
  // ops outside them are launched one by one.
  struct TeamRun {
    int32_t first = 0, count = 0;
    qasr::TeamOp* ops_dev = nullptr;
    qasr::TeamCtl* ctl = nullptr;
  };
  std::vector<TeamRun> runs;
  std::vector<int32_t> run_of;    // per op: index into runs, or -1
  int8_t* toeplitz = nullptr;     // device: Toeplitz operand images of the depthwise layers inside runs
  int32_t team_wgs = 0;           // workgroups of a team launch (one per compute unit)
};


// ---- team runs: which ops one launch of the persistent kernel takes (host logic only until the
// device arrays are filled).  A run is a maximal stretch of consecutive ops whose shapes the team
// kernel's layer bodies take; it needs at least 8 utterances (one per XCD) and 3 ops to pay.
constexpr int32_t kMinRunOps = 3;

static bool team_record(const qasr_encoder::Op& op, qasr::TeamOp& t) {
  if (op.has_act || op.n_more_res > 0) return false;
  t = qasr::TeamOp{};
  const ConvParams& p = op.p;
  if (p.depthwise) {
    if (!qasr::team_dw_geometry(p, t)) return false;
    t.kind = 1;
  } else {
    if (!qasr::team_pw_geometry(p, t)) return false;
    t.kind = 0;
  }
  t.xbs = p.xbs; t.ybs = p.ybs;
  t.Cin = p.Cin; t.Cout = p.Cout; t.T = p.Tin;
  t.relu = p.relu;
  t.w = p.w; t.bias = p.bias; t.m = p.m; t.s = p.s;
  return true;
}

static qasr_status plan_team_runs(qasr_encoder* e, int32_t n_slots) {
  const int32_t n = (int32_t)e->ops.size();
  e->run_of.assign(n, -1);
  if (!qasr::tuning().team || n < kMinRunOps || e->ops[0].d.B < 8 || n > qasr::kTeamMaxStamps - 2) return QASR_OK;
  std::vector<qasr::TeamOp> rec(n);
  std::vector<char> can(n, 0);
  bool any = false;
  for (int32_t i = 0; i < n; ++i) {
    can[i] = team_record(e->ops[i], rec[i]) ? 1 : 0;
    any = any || can[i];
  }
  if (!any) return QASR_OK;
  e->team_wgs = qasr::team_workgroups();        // (first HIP call of the planner)
  if (e->team_wgs <= 0) return QASR_OK;

  // runs, Toeplitz images
  size_t toep_bytes = 0;
  for (int32_t i = 0; i < n;) {
    if (!can[i]) { ++i; continue; }
    int32_t j = i;
    while (j < n && can[j]) ++j;
    if (j - i >= kMinRunOps) {
      qasr_encoder::TeamRun r;
      r.first = i;
      r.count = j - i;
      for (int32_t q = i; q < j; ++q) {
        e->run_of[q] = (int32_t)e->runs.size();
        if (rec[q].kind == 1) toep_bytes += round256(qasr::team_toeplitz_bytes(rec[q], rec[q].Cout));
      }
      e->runs.push_back(r);
    }
    i = j;
  }
  if (e->runs.empty()) return QASR_OK;
  if (toep_bytes) {
    const hipError_t me = hipMalloc((void**)&e->toeplitz, toep_bytes);
    if (me != hipSuccess) return hip_status(me);
  }
  size_t toff = 0;
  for (qasr_encoder::TeamRun& r : e->runs) {
    // a barrier goes before an op that touches what an op since the last barrier wrote, or writes
    // what one of them read (the first op of a run follows a kernel boundary)
    std::vector<char> written(n_slots, 0), read(n_slots, 0);
    for (int32_t q = r.first; q < r.first + r.count; ++q) {
      const qasr_encoder::Op& op = e->ops[q];
      qasr::TeamOp& t = rec[q];
      const bool hazard = written[op.in_slot] || (op.res_slot >= 0 && written[op.res_slot]) ||
                          written[op.out_slot] || read[op.out_slot];
      t.sync_before = hazard ? 1 : 0;
      if (hazard) {
        std::fill(written.begin(), written.end(), 0);
        std::fill(read.begin(), read.end(), 0);
      }
      read[op.in_slot] = 1;
      if (op.res_slot >= 0) read[op.res_slot] = 1;
      written[op.out_slot] = 1;
      // operands: slot 0 is the network input, the last op's output the network output
      t.in_kind = op.in_slot == 0 ? 0 : 1;
      t.in_off = op.in_slot == 0 ? 0 : (int64_t)e->slot_off[op.in_slot];
      t.res_kind = op.res_slot < 0 ? -1 : (op.res_slot == 0 ? 0 : 1);
      t.res_off = op.res_slot <= 0 ? 0 : (int64_t)e->slot_off[op.res_slot];
      t.out_kind = (q + 1 == n) ? 2 : 1;
      t.out_off = (q + 1 == n) ? 0 : (int64_t)e->slot_off[op.out_slot];
      if (t.kind == 1) {
        int8_t* img = e->toeplitz + toff;
        toff += round256(qasr::team_toeplitz_bytes(t, t.Cout));
        const hipError_t te = qasr::launch_toeplitz_image(op.p.w, op.p.Cout, op.p.k, op.p.dil, t, img, nullptr);
        if (te != hipSuccess) return hip_status(te);
        t.w = img;
      }
    }
    hipError_t me = hipMalloc((void**)&r.ops_dev, sizeof(qasr::TeamOp) * (size_t)r.count);
    if (me == hipSuccess) me = hipMalloc((void**)&r.ctl, sizeof(qasr::TeamCtl));
    if (me == hipSuccess)
      me = hipMemcpy(r.ops_dev, rec.data() + r.first, sizeof(qasr::TeamOp) * (size_t)r.count, hipMemcpyHostToDevice);
    if (me == hipSuccess) me = hipMemset(r.ctl, 0, sizeof(qasr::TeamCtl));
    if (me != hipSuccess) return hip_status(me);
  }
  return QASR_OK;
}

extern "C" {

int32_t qasr_conv1d_out_len(const qasr_conv1d_desc* d) {
  const qasr_status st = check_desc(d);
  if (st != QASR_OK) return (int32_t)st;
  return (int32_t)out_len64(d);
}

const char* qasr_conv1d_kernel_name(const qasr_conv1d_desc* d) {
  if (check_desc(d) != QASR_OK) return nullptr;
  const ConvParams p = make_params(d, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  return kernel_name(pick_kernel(p));
}

qasr_status qasr_conv1d_int8(const qasr_conv1d_desc* d, const int8_t* x, const int8_t* w,
                             const int32_t* bias, const int32_t* m, const int32_t* s,
                             const int8_t* residual, int8_t* y, void* stream) {
  const qasr_status st = check_desc(d);
  if (st != QASR_OK) return st;
  if (!x || !w || !m || !s || !y) return QASR_ERR_NULL;
  const ConvParams p = make_params(d, x, w, bias, m, s, residual, y);
  const int64_t ny = (int64_t)(p.B - 1) * p.ybs + (int64_t)p.Cout * p.Tout;
  const int64_t nx = (int64_t)(p.B - 1) * p.xbs + (int64_t)p.Cin * p.Tin;
  if (overlaps(y, ny, x, nx) || (residual && overlaps(y, ny, residual, ny))) return QASR_ERR_ALIAS;
  return launch(p, (hipStream_t)stream);
}

qasr_status qasr_conv1d_int8_multi(const qasr_conv1d_desc* d, const int8_t* x, const int8_t* w,
                                   const int32_t* bias, const int32_t* m, const int32_t* s,
                                   const int8_t* const* residuals, int32_t n_res, int8_t* y, void* stream) {
  const qasr_status st = check_desc(d);
  if (st != QASR_OK) return st;
  if (!x || !w || !m || !s || !y) return QASR_ERR_NULL;
  if (n_res < 0 || n_res > QASR_MAX_RESIDUALS) return QASR_ERR_PARAM;
  if (n_res > 0 && !residuals) return QASR_ERR_NULL;
  for (int32_t r = 0; r < n_res; ++r)
    if (!residuals[r]) return QASR_ERR_NULL;
  ConvParams p = make_params(d, x, w, bias, m, s, n_res > 0 ? residuals[0] : nullptr, y);
  p.n_res_more = n_res > 1 ? n_res - 1 : 0;
  for (int32_t r = 1; r < n_res; ++r) p.res_more[r - 1] = residuals[r];
  const int64_t ny = (int64_t)(p.B - 1) * p.ybs + (int64_t)p.Cout * p.Tout;
  const int64_t nx = (int64_t)(p.B - 1) * p.xbs + (int64_t)p.Cin * p.Tin;
  if (overlaps(y, ny, x, nx)) return QASR_ERR_ALIAS;
  for (int32_t r = 0; r < n_res; ++r)
    if (overlaps(y, ny, residuals[r], ny)) return QASR_ERR_ALIAS;
  return launch(p, (hipStream_t)stream);
}

size_t qasr_packed_weight_bytes(const qasr_conv1d_desc* d) {
  if (check_desc(d) != QASR_OK) return 0;
  return packed_bytes_of(d);
}

qasr_status qasr_pack_weights(const qasr_conv1d_desc* d, const int8_t* w, int8_t* w_packed, void* stream) {
  const qasr_status st = check_desc(d);
  if (st != QASR_OK) return st;
  if (!w || !w_packed) return QASR_ERR_NULL;
  const size_t n = packed_bytes_of(d);
  const int64_t n_plain = (int64_t)d->Cout * (d->groups != 1 ? 1 : d->Cin) * d->k;
  if (overlaps(w, n_plain, w_packed, (int64_t)n)) return QASR_ERR_ALIAS;
  hipError_t e;
  if (!has_packed_form(d))   // packed form == plain form
    e = hipMemcpyAsync(w_packed, w, n, hipMemcpyDeviceToDevice, (hipStream_t)stream);
  else
    e = qasr::launch_pack_weights(w, w_packed, d->Cout, d->Cin, d->k, (hipStream_t)stream);
  return hip_status(e);
}

qasr_status qasr_requant(const int32_t* acc, int32_t B, int32_t C, int32_t T, const int32_t* bias,
                         const int32_t* m, const int32_t* s, const int8_t* residual, uint32_t flags,
                         int8_t* y, void* stream) {
  if (!acc || !m || !s || !y) return QASR_ERR_NULL;
  if (B < 1 || C < 1 || T < 1) return QASR_ERR_SHAPE;
  if (flags & ~(uint32_t)QASR_FLAG_RELU) return QASR_ERR_PARAM;
  const int64_t n = (int64_t)B * C * T;
  if (overlaps(y, n, acc, 4 * n) || (residual && overlaps(y, n, residual, n))) return QASR_ERR_ALIAS;
  const hipError_t e = qasr::launch_requant(acc, B, C, T, bias, m, s, residual,
                                            (flags & QASR_FLAG_RELU) ? 1 : 0, y, (hipStream_t)stream);
  return hip_status(e);
}

qasr_status qasr_quantize(const float* x, size_t n, float alpha, int8_t* q, void* stream) {
  if (!(alpha > 0.0f) || !std::isfinite(alpha)) return QASR_ERR_PARAM;
  const float S = alpha / 127.0f;
  if (!(S > 0.0f)) return QASR_ERR_PARAM;                 // alpha so small that the step underflows
  if (n == 0) return QASR_OK;
  if (!x || !q) return QASR_ERR_NULL;
  if (n > ((size_t)1 << 40)) return QASR_ERR_SHAPE;
  if (overlaps(q, (int64_t)n, x, 4 * (int64_t)n)) return QASR_ERR_ALIAS;
  return hip_status(qasr::launch_quantize(x, n, alpha, S, q, (hipStream_t)stream));
}

qasr_status qasr_dequantize(const int8_t* q, size_t n, float S, float* x, void* stream) {
  if (!std::isfinite(S)) return QASR_ERR_PARAM;
  if (n == 0) return QASR_OK;
  if (!x || !q) return QASR_ERR_NULL;
  if (n > ((size_t)1 << 40)) return QASR_ERR_SHAPE;
  if (overlaps(x, 4 * (int64_t)n, q, (int64_t)n)) return QASR_ERR_ALIAS;
  return hip_status(qasr::launch_dequantize(q, n, S, x, (hipStream_t)stream));
}

qasr_status qasr_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (bytes == 0) return QASR_OK;
  if (!src || !dst) return QASR_ERR_NULL;
  if (bytes % 16 || (uintptr_t)src % 16 || (uintptr_t)dst % 16) return QASR_ERR_SHAPE;
  if (bytes > ((size_t)1 << 40)) return QASR_ERR_SHAPE;
  if (overlaps(dst, (int64_t)bytes, src, (int64_t)bytes)) return QASR_ERR_ALIAS;
  return hip_status(qasr::launch_probe_copy(src, dst, bytes, (hipStream_t)stream));
}

int32_t qasr_probe_mfma_i8_outputs(void) { return qasr::probe_mfma_workgroups(); }

qasr_status qasr_probe_mfma_i8(int32_t iters, int32_t* out, double* ops, void* stream) {
  if (!out || !ops) return QASR_ERR_NULL;
  if (iters < 1 || iters > (1 << 24)) return QASR_ERR_PARAM;
  *ops = qasr::probe_mfma_ops(iters);
  return hip_status(qasr::launch_probe_mfma(iters, out, (hipStream_t)stream));
}

qasr_status qasr_observe_minmax(const float* x, size_t n, float* minmax, void* stream) {
  if (n == 0) return QASR_OK;
  if (!x || !minmax) return QASR_ERR_NULL;
  if (n > ((size_t)1 << 40)) return QASR_ERR_SHAPE;
  if (overlaps(minmax, 8, x, 4 * (int64_t)n)) return QASR_ERR_ALIAS;
  return hip_status(qasr::launch_minmax(x, n, minmax, (hipStream_t)stream));
}

qasr_status qasr_dyadic_from_scale(double M, int32_t* m, int32_t* s) {
  if (!m || !s) return QASR_ERR_NULL;
  int32_t mm, ss;
  if (!qasr::dyadic_from_scale(M, mm, ss)) return QASR_ERR_PARAM;
  *m = mm;
  *s = ss;
  return QASR_OK;
}

qasr_status qasr_fold_bn_quantize(const float* w, const float* conv_bias, const float* gamma, const float* beta,
                                  const float* mean, const float* var, float eps, int32_t Cout, int64_t per_channel,
                                  float S_x, float S_y, int8_t* q_w, int32_t* bias_q, int32_t* m, int32_t* s,
                                  float* S_w, int32_t* bad_count, void* stream) {
  if (!w || !gamma || !beta || !mean || !var || !q_w || !bias_q || !m || !s) return QASR_ERR_NULL;
  if (Cout < 1 || per_channel < 1 || per_channel > ((int64_t)1 << 40) / Cout) return QASR_ERR_SHAPE;
  if (!(S_x > 0.0f) || !std::isfinite(S_x) || !(S_y > 0.0f) || !std::isfinite(S_y) || !(eps >= 0.0f) || !std::isfinite(eps))
    return QASR_ERR_PARAM;
  if (overlaps(q_w, (int64_t)Cout * per_channel, w, 4 * (int64_t)Cout * per_channel)) return QASR_ERR_ALIAS;
  return hip_status(qasr::launch_fold_quantize(w, conv_bias, gamma, beta, mean, var, eps, Cout, per_channel, S_x, S_y, q_w,
                                               bias_q, m, s, S_w, bad_count, (hipStream_t)stream));
}

static qasr_status check_iexp(const qasr_iexp* c) {
  if (!c) return QASR_ERR_NULL;
  if (c->u < 0 || c->u > 16 || c->q_ln2 < 1 || c->q_b < 0 || c->q_b >= ((int64_t)1 << 24) || c->q_c < 0 ||
      c->q_c >= ((int64_t)1 << 48))
    return QASR_ERR_PARAM;
  return QASR_OK;
}

static qasr_status check_act(const qasr_act* a) {
  if (!a) return QASR_ERR_NULL;
  if (a->kind != QASR_ACT_SIGMOID && a->kind != QASR_ACT_SWISH && a->kind != QASR_ACT_GLU) return QASR_ERR_PARAM;
  if (a->m < 0 || a->s < 1 || a->s > 62) return QASR_ERR_PARAM;
  return check_iexp(&a->e);
}

static qasr::ActParams act_params(int32_t kind, int32_t m, int32_t s, const qasr_iexp& e) {
  qasr::ActParams p;
  p.kind = kind; p.m = m; p.s = s; p.u = e.u;
  p.q_ln2 = e.q_ln2; p.q_b = e.q_b; p.q_c = e.q_c;
  return p;
}

qasr_status qasr_iexp_init(double S, int32_t u, qasr_iexp* c) {
  if (!c) return QASR_ERR_NULL;
  if (!(S > 0.0) || !std::isfinite(S) || u < 0 || u > 16) return QASR_ERR_PARAM;
  const double step = std::ldexp(S, -u);                   // S / 2^u, exact
  const double ln2 = 0.6931471805599453;                    // nearest double to ln 2
  const double q_ln2 = std::floor(ln2 / step);
  const double q_b = std::floor(1.353 / step);
  const double q_c = std::floor(0.344 / (0.3585 * step * step));
  if (!(q_ln2 >= 1.0) || !(q_b < 16777216.0)) return QASR_ERR_PARAM;
  c->u = u;
  c->reserved = 0;
  c->q_ln2 = (int64_t)q_ln2;
  c->q_b = (int64_t)q_b;
  c->q_c = (int64_t)q_c;
  return QASR_OK;
}

qasr_status qasr_act_int8(const qasr_act* a, const int8_t* x, int32_t B, int32_t C, int32_t T,
                          int64_t x_batch_stride, int64_t y_batch_stride, int8_t* y, void* stream) {
  const qasr_status st = check_act(a);
  if (st != QASR_OK) return st;
  if (!x || !y) return QASR_ERR_NULL;
  if (B < 1 || B > 65535 || C < 1 || T < 1) return QASR_ERR_SHAPE;
  const int64_t n = (int64_t)C * T, nx = a->kind == QASR_ACT_GLU ? 2 * n : n;
  const int64_t xbs = x_batch_stride ? x_batch_stride : nx, ybs = y_batch_stride ? y_batch_stride : n;
  if (xbs < nx || ybs < n) return QASR_ERR_SHAPE;
  const bool in_place = (const int8_t*)y == x && xbs == ybs;
  if (!in_place && overlaps(y, (int64_t)(B - 1) * ybs + n, x, (int64_t)(B - 1) * xbs + nx)) return QASR_ERR_ALIAS;
  return hip_status(qasr::launch_act(act_params(a->kind, a->m, a->s, a->e), x, y, B, n, xbs, ybs, (hipStream_t)stream));
}

qasr_status qasr_softmax_int32(const qasr_iexp* e, const int32_t* x, int64_t rows, int32_t L, int8_t* y,
                               void* stream) {
  const qasr_status st = check_iexp(e);
  if (st != QASR_OK) return st;
  if (!x || !y) return QASR_ERR_NULL;
  if (rows < 1 || L < 1 || L > 16384 || rows > ((int64_t)1 << 40) / L) return QASR_ERR_SHAPE;
  // the row sum of exponentials (each at most q_b^2 + q_c) times 2^8 must stay inside 64 bits
  if ((double)L * ((double)e->q_b * (double)e->q_b + (double)e->q_c) >= 36028797018963968.0) return QASR_ERR_PARAM;
  if (overlaps(y, rows * L, x, 4 * rows * L)) return QASR_ERR_ALIAS;
  return hip_status(qasr::launch_softmax(act_params(0, 0, 1, *e), x, rows, L, y, (hipStream_t)stream));
}

// ---- buffers for the activation slots.  The caller's slot numbers say which op reads what; which
// memory a value lives in is the library's choice.  It matters: a kernel that writes a buffer which
// the kernel right before it READ runs 3-4 us longer (measured on single layers and on the whole
// encoder: the lines are still held by the L2s of the XCDs that read them, under another
// workgroup-to-XCD mapping, and every write has to displace them), and the two-slot ping-pong of a
// plain layer chain does exactly that in every layer.  So the values are renamed onto physical
// buffers: the output of op i takes the buffer that has been free longest among those that none of
// the `depth` ops before it touched, a new one if there is none (depth + 2 buffers for a plain
// chain).  depth 0 keeps the caller's slots as the buffers.
struct SlotPlan {
  std::vector<int32_t> in, res, out;                 // physical buffer per op (0 = the network input)
  std::vector<std::vector<int32_t>> more;
  std::vector<size_t> bytes;                         // per physical buffer (index 0 unused)
};

struct SlotWire {                                    // what one op reads and writes, in the caller's slots
  int32_t in, res, out;
  std::vector<int32_t> more;
  size_t bytes;                                      // of the value it writes (0: goes to the caller's output)
};

static void plan_slots(const std::vector<SlotWire>& ops, int32_t n_slots, int depth, SlotPlan& pl) {
  const int32_t n_ops = (int32_t)ops.size();
  pl.in.resize(n_ops); pl.res.assign(n_ops, -1); pl.out.resize(n_ops); pl.more.assign(n_ops, {});
  if (depth <= 0) {
    pl.bytes.assign(n_slots, 0);
    for (int32_t i = 0; i < n_ops; ++i) {
      pl.in[i] = ops[i].in; pl.res[i] = ops[i].res; pl.out[i] = ops[i].out;
      pl.more[i] = ops[i].more;
      if (ops[i].bytes > pl.bytes[ops[i].out]) pl.bytes[ops[i].out] = ops[i].bytes;
    }
    return;
  }
  // values: 0 is the network input, i + 1 what op i writes
  std::vector<int32_t> cur(n_slots, -1), last_use(n_ops + 1, -1);
  cur[0] = 0;
  std::vector<std::vector<int32_t>> reads(n_ops);
  for (int32_t i = 0; i < n_ops; ++i) {
    const SlotWire& o = ops[i];
    reads[i].push_back(cur[o.in]);
    if (o.res >= 0) reads[i].push_back(cur[o.res]);
    for (int32_t sl : o.more) reads[i].push_back(cur[sl]);
    for (int32_t v : reads[i]) last_use[v] = i;
    cur[o.out] = i + 1;
  }
  std::vector<int32_t> buf_of(n_ops + 1, -1), holders, free_q;
  buf_of[0] = 0;
  pl.bytes.assign(1, 0);
  std::vector<std::vector<int32_t>> touched(n_ops);
  for (int32_t i = 0; i < n_ops; ++i) {
    for (size_t h = 0; h < holders.size();) {              // values nobody reads from op i on
      if (last_use[holders[h]] < i) {
        free_q.push_back(buf_of[holders[h]]);
        holders.erase(holders.begin() + (long)h);
      } else {
        ++h;
      }
    }
    auto recent = [&](int32_t b) {
      for (int32_t j = i - 1; j >= 0 && j >= i - depth; --j)
        for (int32_t t : touched[j])
          if (t == b) return true;
      return false;
    };
    int32_t b = -1;
    for (size_t q = 0; q < free_q.size(); ++q)
      if (!recent(free_q[q])) {
        b = free_q[q];
        free_q.erase(free_q.begin() + (long)q);
        break;
      }
    if (b < 0) {
      b = (int32_t)pl.bytes.size();
      pl.bytes.push_back(0);
    }
    buf_of[i + 1] = b;
    pl.out[i] = b;
    holders.push_back(i + 1);
    if (ops[i].bytes > pl.bytes[b]) pl.bytes[b] = ops[i].bytes;
    size_t k = 0;
    pl.in[i] = buf_of[reads[i][k++]];
    if (ops[i].res >= 0) pl.res[i] = buf_of[reads[i][k++]];
    for (; k < reads[i].size(); ++k) pl.more[i].push_back(buf_of[reads[i][k]]);
    touched[i].push_back(b);
    for (int32_t v : reads[i]) touched[i].push_back(buf_of[v]);
  }
}

qasr_status qasr_plan_slot_buffers(const int32_t* in_slot, const int32_t* res_slot, const int32_t* out_slot,
                                   int32_t n_ops, int32_t n_slots, int32_t depth, int32_t* in_buf,
                                   int32_t* res_buf, int32_t* out_buf, int32_t* n_buffers) {
  if (!in_slot || !res_slot || !out_slot || !in_buf || !res_buf || !out_buf || !n_buffers) return QASR_ERR_NULL;
  if (n_ops < 1 || n_slots < 2) return QASR_ERR_SHAPE;
  if (depth < 0 || depth > 16) return QASR_ERR_PARAM;
  std::vector<char> live(n_slots, 0);
  live[0] = 1;
  std::vector<SlotWire> w(n_ops);
  for (int32_t i = 0; i < n_ops; ++i) {
    if (in_slot[i] < 0 || in_slot[i] >= n_slots || out_slot[i] < 1 || out_slot[i] >= n_slots || res_slot[i] < -1 ||
        res_slot[i] >= n_slots || out_slot[i] == in_slot[i] || out_slot[i] == res_slot[i])
      return QASR_ERR_PARAM;
    if (!live[in_slot[i]] || (res_slot[i] >= 0 && !live[res_slot[i]])) return QASR_ERR_PARAM;
    live[out_slot[i]] = 1;
    w[i] = SlotWire{in_slot[i], res_slot[i], out_slot[i], {}, (size_t)1};
  }
  SlotPlan pl;
  plan_slots(w, n_slots, depth, pl);
  for (int32_t i = 0; i < n_ops; ++i) { in_buf[i] = pl.in[i]; res_buf[i] = pl.res[i]; out_buf[i] = pl.out[i]; }
  *n_buffers = (int32_t)pl.bytes.size();
  return QASR_OK;
}

qasr_status qasr_encoder_create(const qasr_op* ops, int32_t n_ops, int32_t n_slots, qasr_encoder** out) {
  if (!ops || !out) return QASR_ERR_NULL;
  if (n_ops < 1 || n_slots < 2) return QASR_ERR_SHAPE;
  *out = nullptr;

  // ---- validation: host only, no HIP call yet
  struct SlotState { bool live = false; int32_t C = 0, T = 0; };
  std::vector<SlotState> slot(n_slots);
  size_t packed_bytes = 0;
  for (int32_t i = 0; i < n_ops; ++i) {
    const qasr_op& o = ops[i];
    const qasr_status st = check_desc(&o.d);
    if (st != QASR_OK) return st;
    if (!o.w || !o.m || !o.s) return QASR_ERR_NULL;
    if (o.d.flags & QASR_FLAG_W_PACKED) return QASR_ERR_PARAM;
    if (o.d.y_batch_stride != 0) return QASR_ERR_PARAM;
    if (o.d.B != ops[0].d.B) return QASR_ERR_SHAPE;
    if (o.in_slot < 0 || o.in_slot >= n_slots || o.out_slot < 1 || o.out_slot >= n_slots ||
        o.res_slot < -1 || o.res_slot >= n_slots)
      return QASR_ERR_PARAM;
    if (o.out_slot == o.in_slot || o.out_slot == o.res_slot) return QASR_ERR_PARAM;
    if (o.n_more_res < 0 || o.n_more_res > QASR_MAX_RESIDUALS - 1 || (o.n_more_res > 0 && o.res_slot < 0))
      return QASR_ERR_PARAM;
    for (int32_t r = 0; r < o.n_more_res; ++r) {
      const int32_t sl = o.more_res_slots[r];
      if (sl < 0 || sl >= n_slots || sl == o.out_slot) return QASR_ERR_PARAM;
    }
    if (o.act) {
      const qasr_status as = check_act(o.act);
      if (as != QASR_OK) return as;
      if (o.act->kind == QASR_ACT_GLU && (o.d.Cout & 1)) return QASR_ERR_SHAPE;
      if (o.d.B > 65535) return QASR_ERR_SHAPE;
    }
    if (i == 0) {
      if (ops[0].in_slot != 0) return QASR_ERR_PARAM;
      slot[0].live = true;
      slot[0].T = o.d.Tin;
      slot[0].C = o.d.x_batch_stride ? (int32_t)(o.d.x_batch_stride / o.d.Tin) : o.d.Cin;
    }
    const SlotState& in = slot[o.in_slot];
    if (!in.live || in.T != o.d.Tin) return QASR_ERR_PARAM;
    if (o.d.x_batch_stride == 0 ? in.C != o.d.Cin
                                : (o.d.x_batch_stride != (int64_t)in.C * in.T || o.d.Cin > in.C))
      return QASR_ERR_PARAM;
    const int32_t Tout = (int32_t)out_len64(&o.d);
    if (o.res_slot >= 0) {
      const SlotState& r = slot[o.res_slot];
      if (!r.live || r.C != o.d.Cout || r.T != Tout) return QASR_ERR_PARAM;
    }
    for (int32_t q = 0; q < o.n_more_res; ++q) {
      const SlotState& r = slot[o.more_res_slots[q]];
      if (!r.live || r.C != o.d.Cout || r.T != Tout) return QASR_ERR_PARAM;
    }
    slot[o.out_slot].live = true;
    slot[o.out_slot].C = o.d.Cout;
    slot[o.out_slot].T = Tout;
    if (has_packed_form(&o.d)) packed_bytes += round256(packed_bytes_of(&o.d));
    if (o.act && o.act->kind != QASR_ACT_GLU) packed_bytes += 256;   // room for a fused activation's table
  }

  qasr_encoder* e = new (std::nothrow) qasr_encoder();
  if (!e) return QASR_ERR_HIP;
  SlotPlan plan;
  {
    std::vector<SlotWire> wires(n_ops);
    for (int32_t i = 0; i < n_ops; ++i) {
      const qasr_op& o = ops[i];
      wires[i] = SlotWire{o.in_slot, o.res_slot, o.out_slot,
                          std::vector<int32_t>(o.more_res_slots, o.more_res_slots + o.n_more_res),
                          i + 1 == n_ops ? (size_t)0   // (the last op writes the caller's output)
                                         : (size_t)o.d.B * o.d.Cout * (size_t)out_len64(&o.d)};
    }
    // The buffers should stay inside the 256 MB memory-side cache together: the deepest plan up to
    // the configured depth whose buffers take at most three quarters of it (QuartzNet-15x5 shape:
    // depth 4 at batch 32, 118 MB; depth 2 at batch 64, 2.44 against 2.46 ms with depth 4 and 2.60
    // with the slots as buffers; at batch 128 even those take 264 MB and every further buffer
    // costs: 4.78 ms with depth 0, 4.92 with 1, 5.53 with 4).
    const size_t budget = (size_t)192 << 20;
    for (int depth = qasr::tuning().slot_depth; depth >= 0; --depth) {
      plan_slots(wires, n_slots, depth, plan);
      size_t total = 0;
      for (size_t b = 1; b < plan.bytes.size(); ++b) total += round256(plan.bytes[b]);
      if (total <= budget) break;
    }
  }
  const int32_t n_bufs = (int32_t)plan.bytes.size();
  e->slot_off.assign(n_bufs, 0);
  size_t off = 0;
  for (int32_t sidx = 1; sidx < n_bufs; ++sidx) {
    e->slot_off[sidx] = off;
    off += round256(plan.bytes[sidx]);
  }
  e->ws_bytes = off;
  e->in_elems = (size_t)ops[0].d.B * slot[0].C * slot[0].T;
  {
    const qasr_conv1d_desc& ld = ops[n_ops - 1].d;
    e->out_elems = (size_t)ld.B * ld.Cout * (size_t)out_len64(&ld);
  }

  // ---- one-time device work: pack the dense k>1 weights
  if (packed_bytes) {
    const hipError_t me = hipMalloc((void**)&e->packed, packed_bytes);
    if (me != hipSuccess) { delete e; return hip_status(me); }
  }
  size_t poff = 0;
  e->ops.resize(n_ops);
  for (int32_t i = 0; i < n_ops; ++i) {
    const qasr_op& o = ops[i];
    qasr_encoder::Op& op = e->ops[i];
    op.d = o.d;
    op.in_slot = plan.in[i]; op.res_slot = plan.res[i]; op.out_slot = plan.out[i];   // (buffers, not the caller's slots)
    const int8_t* w = o.w;
    if (has_packed_form(&o.d)) {
      int8_t* wp = e->packed + poff;
      poff += round256(packed_bytes_of(&o.d));
      const hipError_t pe = qasr::launch_pack_weights(o.w, wp, o.d.Cout, o.d.Cin, o.d.k, nullptr);
      if (pe != hipSuccess) {
        qasr_encoder_destroy(e);
        return hip_status(pe);
      }
      w = wp;
      op.d.flags |= QASR_FLAG_W_PACKED;
    }
    op.p = make_params(&op.d, nullptr, w, o.bias, o.m, o.s, nullptr, nullptr);
    op.n_more_res = o.n_more_res;
    op.p.n_res_more = o.n_more_res;
    for (int32_t r = 0; r < o.n_more_res; ++r) op.more_res_slots[r] = plan.more[i][r];
    op.kernel = pick_kernel(op.p);
    if (o.act) {
      op.has_act = true;
      op.act = act_params(o.act->kind, o.act->m, o.act->s, o.act->e);
      // A unary activation after a layer of the pipelined pointwise or depthwise kernel is applied in
      // that kernel's epilogue through a 256-entry table (one int8 output per int8 code), built here
      // once by the activation's own integer arithmetic; everything else keeps the separate pass.
      if (o.act->kind != QASR_ACT_GLU) {
        uint8_t* table = reinterpret_cast<uint8_t*>(e->packed + poff);
        poff += 256;
        if (applies_act_table(op.kernel)) {
          const hipError_t te = qasr::launch_act_table(op.act, table, nullptr);
          if (te != hipSuccess) {
            qasr_encoder_destroy(e);
            return hip_status(te);
          }
          op.p.act_lut = table;
          op.act_fused = true;
        }
      }
    }
  }
  {
    const qasr_status ts = plan_team_runs(e, n_bufs);
    if (ts != QASR_OK) {
      qasr_encoder_destroy(e);
      return ts;
    }
  }
  if (packed_bytes || !e->runs.empty()) {
    const hipError_t se = hipStreamSynchronize(nullptr);
    if (se != hipSuccess) {
      qasr_encoder_destroy(e);
      return hip_status(se);
    }
  }
  *out = e;
  return QASR_OK;
}

size_t qasr_encoder_workspace_bytes(const qasr_encoder* e) { return e ? e->ws_bytes : 0; }

int32_t qasr_encoder_num_ops(const qasr_encoder* e) { return e ? (int32_t)e->ops.size() : 0; }

const char* qasr_encoder_op_kernel(const qasr_encoder* e, int32_t i) {
  if (!e || i < 0 || i >= (int32_t)e->ops.size()) return nullptr;
  return kernel_name(e->ops[i].kernel);
}

int32_t qasr_encoder_op_act_fused(const qasr_encoder* e, int32_t i) {
  if (!e || i < 0 || i >= (int32_t)e->ops.size()) return -1;
  return e->ops[i].act_fused ? 1 : 0;
}

// team: 0 = every op as a launch of its own, 1 = the planned runs through the team kernel,
// 2 = the same with the team kernel's per-layer clock stamps switched on
int32_t qasr_encoder_op_in_team(const qasr_encoder* e, int32_t i) {
  if (!e || i < 0 || i >= (int32_t)e->ops.size()) return -1;
  return e->run_of.empty() ? 0 : (e->run_of[i] >= 0 ? 1 : 0);
}

static qasr_status forward_impl(const qasr_encoder* e, const int8_t* x, int8_t* y, void* workspace,
                                size_t workspace_bytes, hipStream_t st, hipEvent_t* ev, int team = 1) {
  if (!e || !x || !y) return QASR_ERR_NULL;
  if (e->ws_bytes && (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < e->ws_bytes))
    return QASR_ERR_WORKSPACE;
  int8_t* ws = (int8_t*)workspace;
  const size_t n = e->ops.size();
  // (the team kernel's loads want 16-byte aligned tensors, like the kernels it replaces)
  const bool use_team = team && !ev && !e->runs.empty() && ((uintptr_t)x % 16 == 0) && ((uintptr_t)y % 16 == 0);
  for (size_t i = 0; i < n; ++i) {
    if (use_team && e->run_of[i] >= 0) {
      const qasr_encoder::TeamRun& r = e->runs[e->run_of[i]];
      const hipError_t te = qasr::launch_team(r.ops_dev, r.count, x, ws, y, e->ops[0].d.B, r.ctl, e->team_wgs,
                                              team == 2 ? 1 : 0, st);
      if (te != hipSuccess) return hip_status(te);
      i = (size_t)(r.first + r.count) - 1;
      continue;
    }
    const qasr_encoder::Op& op = e->ops[i];
    ConvParams p = op.p;
    p.x = op.in_slot == 0 ? x : ws + e->slot_off[op.in_slot];
    p.res = op.res_slot < 0 ? nullptr : (op.res_slot == 0 ? x : ws + e->slot_off[op.res_slot]);
    p.y = (i + 1 == n) ? y : ws + e->slot_off[op.out_slot];
    for (int32_t r = 0; r < op.n_more_res; ++r)
      p.res_more[r] = op.more_res_slots[r] == 0 ? x : ws + e->slot_off[op.more_res_slots[r]];
    if (ev) { const hipError_t re = hipEventRecord(ev[i], st); if (re != hipSuccess) return hip_status(re); }
    // (the choice depends on the caller's pointers too: a fused activation's table is only read
    // by the two pipelined kernels, any other choice is followed by the separate pass)
    const Kernel kk = pick_kernel(p);
    const qasr_status s = launch_with(kk, p, st);
    if (s != QASR_OK) return s;
    if (op.has_act && !(op.act_fused && applies_act_table(kk))) {
      const bool glu = op.act.kind == QASR_ACT_GLU;
      const int64_t n_out = (int64_t)(glu ? p.Cout / 2 : p.Cout) * p.Tout;
      const hipError_t ae = qasr::launch_act(op.act, p.y, p.y, p.B, n_out, p.ybs, p.ybs, st);
      if (ae != hipSuccess) return hip_status(ae);
    }
  }
  if (ev) { const hipError_t re = hipEventRecord(ev[n], st); if (re != hipSuccess) return hip_status(re); }
  return QASR_OK;
}

qasr_status qasr_encoder_forward(const qasr_encoder* e, const int8_t* x, int8_t* y, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  return forward_impl(e, x, y, workspace, workspace_bytes, (hipStream_t)stream, nullptr);
}

// ---- the forward for callers that can neither allocate nor pass a workspace: the activation slots
// live in a static device array of the library.  The array's name is only a host-side stand-in; its
// device address is looked up once per device and kept.
#define QASR_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
static __device__ __align__(256) unsigned char scratch[QASR_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up at the first call on that device)
qasr_status static_scratch(void** out) {
  int dev = 0;
  const hipError_t ge = hipGetDevice(&dev);
  if (ge != hipSuccess) return hip_status(ge);
  if (dev < 0 || dev >= kMaxDevices) return QASR_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t se = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (se != hipSuccess) return hip_status(se);
    if (!ptr || ((uintptr_t)ptr & 255)) return QASR_ERR_WORKSPACE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return QASR_OK;
}

}  // namespace

size_t qasr_static_workspace_bytes(void) { return QASR_STATIC_WORKSPACE_BYTES; }

qasr_status qasr_encoder_forward_static(const qasr_encoder* e, const int8_t* x, int8_t* y, void* stream) {
  if (!e || !x || !y) return QASR_ERR_NULL;
  if (e->ws_bytes > QASR_STATIC_WORKSPACE_BYTES) return QASR_ERR_WORKSPACE;     // before any HIP call
  void* ws = nullptr;
  const qasr_status st = static_scratch(&ws);
  if (st != QASR_OK) return st;
  // every slot is written in full by the op that produces it before any op reads it: nothing in the
  // array has to start at zero, whatever an earlier call left there
  return forward_impl(e, x, y, ws, QASR_STATIC_WORKSPACE_BYTES, (hipStream_t)stream, nullptr);
}

qasr_status qasr_encoder_forward_layerwise(const qasr_encoder* e, const int8_t* x, int8_t* y, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  return forward_impl(e, x, y, workspace, workspace_bytes, (hipStream_t)stream, nullptr, 0);
}

qasr_status qasr_encoder_team_check(const qasr_encoder* e, int32_t* aborted) {
  if (!e || !aborted) return QASR_ERR_NULL;
  *aborted = 0;
  for (const qasr_encoder::TeamRun& r : e->runs) {
    uint32_t flag = 0;
    const hipError_t ce = hipMemcpy(&flag, &r.ctl->abort, sizeof(flag), hipMemcpyDeviceToHost);
    if (ce != hipSuccess) return hip_status(ce);
    if (flag) *aborted = 1;
  }
  return QASR_OK;
}

qasr_status qasr_encoder_forward_team_stamps(const qasr_encoder* e, const int8_t* x, int8_t* y, void* workspace,
                                             size_t workspace_bytes, void* stream, float* op_us) {
  if (!e || !op_us) return QASR_ERR_NULL;
  const size_t n = e->ops.size();
  for (size_t i = 0; i < n; ++i) op_us[i] = 0.f;
  qasr_status st = forward_impl(e, x, y, workspace, workspace_bytes, (hipStream_t)stream, nullptr, 2);
  if (st != QASR_OK) return st;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return QASR_ERR_HIP;
  std::vector<unsigned long long> stamp(qasr::kTeamMaxStamps);
  for (const qasr_encoder::TeamRun& r : e->runs) {
    const hipError_t ce = hipMemcpy(stamp.data(), r.ctl->stamp, sizeof(unsigned long long) * (size_t)(r.count + 1),
                                    hipMemcpyDeviceToHost);
    if (ce != hipSuccess) return hip_status(ce);
    for (int32_t q = 0; q < r.count; ++q)       // the clock runs at 100 MHz
      op_us[r.first + q] = (float)((double)(stamp[q + 1] - stamp[q]) * 0.01);
  }
  return st;
}

size_t qasr_encoder_workspace_bytes_f32(const qasr_encoder* e) {
  return e ? e->ws_bytes + round256(e->in_elems) + round256(e->out_elems) : 0;
}

qasr_status qasr_encoder_forward_f32(const qasr_encoder* e, const float* x, float alpha, float S_out, float* y,
                                     void* workspace, size_t workspace_bytes, void* stream) {
  if (!e || !x || !y) return QASR_ERR_NULL;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < qasr_encoder_workspace_bytes_f32(e))
    return QASR_ERR_WORKSPACE;
  int8_t* xq = (int8_t*)workspace + e->ws_bytes;
  int8_t* yq = xq + round256(e->in_elems);
  qasr_status st = qasr_quantize(x, e->in_elems, alpha, xq, stream);
  if (st == QASR_OK) st = forward_impl(e, xq, yq, workspace, e->ws_bytes ? e->ws_bytes : workspace_bytes, (hipStream_t)stream, nullptr);
  if (st == QASR_OK) st = qasr_dequantize(yq, e->out_elems, S_out, y, stream);
  return st;
}

qasr_status qasr_encoder_forward_timed(const qasr_encoder* e, const int8_t* x, int8_t* y, void* workspace,
                                       size_t workspace_bytes, void* stream, float* op_ms) {
  if (!e || !op_ms) return QASR_ERR_NULL;
  const size_t n = e->ops.size();
  std::vector<hipEvent_t> ev(n + 1, nullptr);
  hipEvent_t cal[2] = {nullptr, nullptr};
  qasr_status st = QASR_OK;
  for (size_t i = 0; i <= n && st == QASR_OK; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) st = QASR_ERR_HIP;
  for (int i = 0; i < 2 && st == QASR_OK; ++i)
    if (hipEventCreate(&cal[i]) != hipSuccess) st = QASR_ERR_HIP;
  // An event record between two kernels costs device time of its own.  The same forward is run
  // once without inner events (bracketed by two) and once with them; the difference of the two
  // totals, spread evenly, is taken off every op's interval, so that the op times add up to the
  // duration of the undisturbed forward.
  if (st == QASR_OK && hipEventRecord(cal[0], (hipStream_t)stream) != hipSuccess) st = QASR_ERR_HIP;
  if (st == QASR_OK) st = forward_impl(e, x, y, workspace, workspace_bytes, (hipStream_t)stream, nullptr, 0);
  if (st == QASR_OK && hipEventRecord(cal[1], (hipStream_t)stream) != hipSuccess) st = QASR_ERR_HIP;
  if (st == QASR_OK) st = forward_impl(e, x, y, workspace, workspace_bytes, (hipStream_t)stream, ev.data());
  if (st == QASR_OK && hipEventSynchronize(ev[n]) != hipSuccess) st = QASR_ERR_HIP;
  float per_event_ms = 0.f;
  if (st == QASR_OK && n > 0) {
    float plain = 0.f, evented = 0.f;
    if (hipEventElapsedTime(&plain, cal[0], cal[1]) != hipSuccess || hipEventElapsedTime(&evented, ev[0], ev[n]) != hipSuccess)
      st = QASR_ERR_HIP;
    per_event_ms = evented > plain ? (evented - plain) / (float)n : 0.f;
  }
  for (size_t i = 0; i < n && st == QASR_OK; ++i) {
    if (hipEventElapsedTime(&op_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = QASR_ERR_HIP;
    op_ms[i] = op_ms[i] > per_event_ms ? op_ms[i] - per_event_ms : 0.f;
  }
  for (hipEvent_t v : cal)
    if (v) (void)hipEventDestroy(v);
  for (hipEvent_t v : ev)
    if (v) (void)hipEventDestroy(v);
  return st;
}

struct qasr_encoder_graph {
  hipGraphExec_t exec = nullptr;
};

qasr_status qasr_encoder_graph_create(const qasr_encoder* e, const int8_t* x, int8_t* y, void* workspace,
                                      size_t workspace_bytes, qasr_encoder_graph** out) {
  if (!e || !out) return QASR_ERR_NULL;
  *out = nullptr;
  hipStream_t cap = nullptr;
  if (hipStreamCreate(&cap) != hipSuccess) return QASR_ERR_HIP;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  // One ordinary forward first: argument checks, and the one-time per-kernel set-up (attribute
  // calls) that must not happen while the stream is capturing.
  qasr_status st = forward_impl(e, x, y, workspace, workspace_bytes, cap, nullptr);
  if (st == QASR_OK && hipStreamSynchronize(cap) != hipSuccess) st = QASR_ERR_HIP;
  if (st == QASR_OK) {
    if (hipStreamBeginCapture(cap, hipStreamCaptureModeThreadLocal) != hipSuccess) {
      st = QASR_ERR_HIP;
    } else {
      st = forward_impl(e, x, y, workspace, workspace_bytes, cap, nullptr);
      const hipError_t ee = hipStreamEndCapture(cap, &graph);      // always ends the capture
      if (st == QASR_OK && (ee != hipSuccess || !graph)) st = QASR_ERR_HIP;
    }
  }
  if (st == QASR_OK && hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess) st = QASR_ERR_HIP;
  if (graph) (void)hipGraphDestroy(graph);
  (void)hipStreamDestroy(cap);
  if (st != QASR_OK) return st;
  qasr_encoder_graph* g = new (std::nothrow) qasr_encoder_graph();
  if (!g) { (void)hipGraphExecDestroy(exec); return QASR_ERR_HIP; }
  g->exec = exec;
  *out = g;
  return QASR_OK;
}

qasr_status qasr_encoder_graph_launch(qasr_encoder_graph* g, void* stream) {
  if (!g || !g->exec) return QASR_ERR_NULL;
  const hipError_t e = hipGraphLaunch(g->exec, (hipStream_t)stream);
  return e == hipSuccess ? QASR_OK : hip_status(e);
}

void qasr_encoder_graph_destroy(qasr_encoder_graph* g) {
  if (!g) return;
  if (g->exec) (void)hipGraphExecDestroy(g->exec);
  delete g;
}

void qasr_encoder_destroy(qasr_encoder* e) {
  if (!e) return;
  if (e->packed) (void)hipFree(e->packed);
  if (e->toeplitz) (void)hipFree(e->toeplitz);
  for (qasr_encoder::TeamRun& r : e->runs) {
    if (r.ops_dev) (void)hipFree(r.ops_dev);
    if (r.ctl) (void)hipFree(r.ctl);
  }
  delete e;
}

void qasr_tuning_reload(void) { qasr::tuning_reload(); }

const char* qasr_last_hip_error(void) { return hipGetErrorName(g_last_hip); }

const char* qasr_status_string(qasr_status st) {
  switch (st) {
    case QASR_OK: return "ok";
    case QASR_ERR_NULL: return "required pointer is NULL";
    case QASR_ERR_SHAPE: return "invalid shape";
    case QASR_ERR_PARAM: return "invalid parameter";
    case QASR_ERR_UNSUPPORTED: return "unsupported grouping";
    case QASR_ERR_ALIAS: return "output overlaps an input";
    case QASR_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case QASR_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

}  // extern "C"
