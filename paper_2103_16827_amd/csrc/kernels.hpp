// Host-callable launchers of the HIP kernels (one translation unit each).
#pragma once
#include "common.hpp"

namespace qasr {

// Generic direct convolution: any stride / dilation / padding / channel count, dense or
// depthwise.  One thread per output element.  The fallback for geometries the MFMA kernels
// do not take.
hipError_t launch_conv_generic(const ConvParams& p, hipStream_t st);

// Standalone epilogue on int32 accumulators.
hipError_t launch_requant(const int32_t* acc, int B, int C, int T, const int32_t* bias,
                          const int32_t* m, const int32_t* s, const int8_t* res, int relu,
                          int8_t* y, hipStream_t st);

// [Cout][Cin][k] -> MFMA operand order (common.hpp: packed_weight_index); needs Cin % 64 == 0
hipError_t launch_pack_weights(const int8_t* w, int8_t* wp, int Cout, int Cin, int k, hipStream_t st);

// Depthwise convolution as a banded-Toeplitz product on the int8 matrix cores (stride 1).
bool dw_mfma_supported(const ConvParams& p);
hipError_t launch_dw_mfma(const ConvParams& p, hipStream_t st);

// Pointwise / dense convolution as an implicit GEMM on the int8 matrix cores.
bool gemm_mfma_supported(const ConvParams& p);
hipError_t launch_gemm_mfma(const ConvParams& p, hipStream_t st);

// Depthwise convolution, same arithmetic, software-pipelined over the batch (reads and writes of
// HBM overlap); needs aligned rows, no residual and enough rows per wave to pipeline.
bool dw_pipe_supported(const ConvParams& p);
hipError_t launch_dw_pipe(const ConvParams& p, hipStream_t st);

// Pointwise convolution (k = 1), activation tile stationary in LDS (direct global->LDS loads);
// needs packed weights, rows that are a multiple of 16 frames and Cin <= 1024.
bool pw_tile_supported(const ConvParams& p);
hipError_t launch_pw_tile(const ConvParams& p, hipStream_t st);

// Pointwise convolution (k = 1), activation tile stationary in LDS, output channels in passes of
// 256 whose epilogues run in between the matrix products of the following pass; needs packed
// weights, rows that are a multiple of 16 frames, Cin in {256, 512} and 256 <= Cout <= 2048.
bool pw_pipe_supported(const ConvParams& p);
hipError_t launch_pw_pipe(const ConvParams& p, hipStream_t st);

// Dense convolution (k >= 2) as an implicit GEMM pipelined over (chunk, tap) steps; needs packed
// weights, Cin % 64 == 0, Cout >= 64, frame counts and strides that are multiples of 4.
bool conv_pipe_supported(const ConvParams& p);
hipError_t launch_conv_pipe(const ConvParams& p, hipStream_t st);

// Measured ceilings (probe.hip): a streaming copy of `bytes` (a multiple of 16) and a register-resident
// int8 matrix-core loop of probe_mfma_ops(iters) operations that writes probe_mfma_workgroups() int32.
hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
int probe_mfma_workgroups();
double probe_mfma_ops(int iters);
hipError_t launch_probe_mfma(int iters, int32_t* out, hipStream_t st);

// Quantiser (Eq. 1, b = 8; S = alpha / 127 from the host) and dequantiser (S * q) at the two ends
// of the path; n elements, any alignment.
hipError_t launch_quantize(const float* x, size_t n, float alpha, float S, int8_t* q, hipStream_t st);
hipError_t launch_dequantize(const int8_t* q, size_t n, float S, float* x, hipStream_t st);

// Integer-only activations (Sec. 2.2: second-order polynomial exponential).  kind 1 sigmoid,
// 2 swish, 3 GLU; u refines an int8 code to scale S / 2^u; q_ln2, q_b, q_c are the host-side
// constants of the exponential at that scale; (m, s) the dyadic rescale of the result.
struct ActParams {
  int32_t kind, m, s, u;
  int64_t q_ln2, q_b, q_c;
};
// x: B items of n (2 n for GLU: value half, gate half) int8 at stride xbs; y: B items of n int8
// at stride ybs; y may be x itself when the strides are equal.
// table[code + 128] = int8 output of the unary activation (sigmoid, swish) for every int8 code
hipError_t launch_act_table(const ActParams& c, uint8_t* table, hipStream_t st);
hipError_t launch_act(const ActParams& c, const int8_t* x, int8_t* y, int32_t B, int64_t n, int64_t xbs,
                      int64_t ybs, hipStream_t st);
// rows x L int32 logits -> int8 probabilities at scale 2^-7 (kind, m, s unused).
hipError_t launch_softmax(const ActParams& c, const int32_t* x, int64_t rows, int32_t L, int8_t* y, hipStream_t st);

// Offline calibration helpers (Sec. 2.1, 2.2, 3.1): running (min, max) of float32 values into
// mm[0..1] (device); the dyadic form of a positive multiplier (host or device arithmetic, the
// same function); BatchNorm folding + per-channel weight quantisation + bias and (m, s).
hipError_t launch_minmax(const float* x, size_t n, float* mm, hipStream_t st);
bool dyadic_from_scale(double M, int32_t& m, int32_t& s);
hipError_t launch_fold_quantize(const float* w, const float* b, const float* gamma, const float* beta, const float* mean,
                                const float* var, float eps, int32_t Cout, int64_t per, float S_x, float S_y, int8_t* qw,
                                int32_t* bias_q, int32_t* m, int32_t* s, float* S_w, int32_t* bad_count, hipStream_t st);

}  // namespace qasr
