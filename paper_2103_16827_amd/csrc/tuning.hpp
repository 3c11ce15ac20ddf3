// Tuning overrides of the kernel choices, read from the environment ONCE (at first use) instead of
// on every launch; tuning_reload() reads them again (tests and sweeps that change the environment
// of a running process call it through qasr_tuning_reload).  0 / false = no override.
//   QASR_NO_PW_PIPE, QASR_NO_CONV_PIPE      fall through to the next kernel family
//   QASR_PWP_MT, QASR_PWP_SPLIT             pw_pipe: groups per tile, workgroups per tile
//   QASR_DWP = "R,S"                        dw_pipe: rows per iteration, batch splits
//   QASR_DW_R                               dw_mfma: strips per wave
//   QASR_CP_TILE = "MT,NT"                  conv_pipe: tile
//   QASR_CP_PLAIN_ORDER                     conv_pipe: tile = workgroup index (no per-XCD runs of the channel-major order)
//   QASR_PWT_MT                             pw_tile: groups per tile
//   QASR_PWP_NOPIPE                         pw_pipe: no epilogue under the next pass's products
//   QASR_PW_LEAN                            pw_pipe: the lean form for every layer it can take, whatever the launch size
//   QASR_PW_LEAN_NO_RES                     pw_pipe: layers with a residual operand keep the pipelined form
//   QASR_NO_PW_LEAN                         pw_pipe: never the lean form (one pass per workgroup, two workgroups per unit)
//   QASR_SLOT_DEPTH                         encoder: an op's output avoids the buffers the last N ops touched
//                                           (default 4; 0 = the caller's slots are the buffers)
//   QASR_TEAM                               encoder: plan runs of layers for the persistent team kernel
//                                           (experimental, off unless set)
#pragma once

namespace qasr {

struct Tuning {
  bool no_pw_pipe = false, no_conv_pipe = false, team = false, cp_plain_order = false, no_pw_lean = false, pw_lean_force = false, pw_lean_no_res = false, pwp_nopipe = false;
  int pwp_mt = 0, pwp_split = 0;
  int dwp_r = 0, dwp_s = 0;
  int dw_r = 0;
  int cp_mt = 0, cp_nt = 0;
  int pwt_mt = 0;
  int slot_depth = 4;
};

const Tuning& tuning();
void tuning_reload();

}  // namespace qasr
