// The persistent team kernel (team.hip): layer records, control block, host entry points.
#pragma once
#include "common.hpp"

namespace qasr {

constexpr int kTeamMaxStamps = 512;

// One layer of a run that the team kernel executes (device memory, read-only while it runs).
struct TeamOp {
  int32_t kind;              // 0 pointwise (the tile of the pipelined pointwise kernel), 1 depthwise
  int32_t sync_before;       // 1: a team barrier precedes this layer (it touches what a layer since the last barrier wrote or read)
  int32_t in_kind, res_kind, out_kind;   // buffer of each operand: 0 network input, 1 workspace, 2 network output; -1 none
  int32_t variant;           // pointwise: Cin / 64 (4 or 8); depthwise: KC, 64-wide chunks of the Toeplitz operand (1..3)
  int64_t in_off, res_off, out_off;      // byte offset of batch item 0 inside that buffer
  int64_t xbs, ybs;          // batch strides (elements) of input and output / residual
  int32_t Cin, Cout, T;      // frames per row (stride 1: Tin == Tout)
  int32_t relu;
  const int8_t* w;           // pointwise: packed weights; depthwise: Toeplitz operand images [C][KC][64 lanes][16 B]
  const int32_t* bias;       // or null
  const int32_t* m;
  const int32_t* s;
  int32_t delta, PH, NCH, G, KC, pad_;   // depthwise geometry (see team.hip)
};

// Control block of one launch (device memory, cleared by a small kernel before every launch).
struct TeamCtl {
  uint32_t registered;       // workgroups that have joined a team
  uint32_t abort;            // a wait was abandoned: everybody leaves
  uint32_t pad0[2];
  uint32_t team_n[16];       // members per XCC id
  uint32_t pad1[12];
  uint32_t team_count[16 * 32];   // barrier counter of each team, 128 bytes apart
  unsigned long long stamp[kTeamMaxStamps];   // wall clock (100 MHz): [0] when the teams stand, [i + 1] after layer i, by team 0's first workgroup (when asked for)
};

// Shape checks (host only) and geometry of a layer inside a team run.
bool team_pw_geometry(const ConvParams& p, TeamOp& t);
bool team_dw_geometry(const ConvParams& p, TeamOp& t);
size_t team_toeplitz_bytes(const TeamOp& t, int C);
// Toeplitz operand images of a depthwise layer's weights [C][k] (once, when the encoder is created)
hipError_t launch_toeplitz_image(const int8_t* w, int C, int k, int dil, const TeamOp& t, int8_t* out, hipStream_t st);
// Workgroups to launch (one per compute unit), 0 if the kernel cannot be resident on every unit.
int team_workgroups();
// Clears the control block (a kernel) and launches the run.  stamps: device array of kTeamMaxStamps
// clock values or null.
hipError_t launch_team(const TeamOp* ops_dev, int n_ops, const int8_t* x, int8_t* ws, int8_t* y, int B, TeamCtl* ctl,
                       int n_workgroups, int stamps_on, hipStream_t st);

}  // namespace qasr
