// Generic direct int8 convolution with the fused epilogue: one thread per output element.
// Takes every geometry the ABI allows; used when the matrix-core kernels do not apply.
#include "kernels.hpp"

namespace qasr {

__global__ __launch_bounds__(256) void conv_generic_kernel(ConvParams p) {
  const int64_t total = (int64_t)p.B * p.Cout * p.Tout;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int to = (int)(idx % p.Tout);
  const int co = (int)((idx / p.Tout) % p.Cout);
  const int b = (int)(idx / ((int64_t)p.Tout * p.Cout));

  int32_t A = p.bias ? p.bias[co] : 0;
  const int8_t* xb = p.x + (int64_t)b * p.xbs;
  const int t0 = to * p.stride - p.pl;
  if (p.depthwise) {
    const int8_t* xr = xb + (int64_t)co * p.Tin;
    const int8_t* wr = p.w + (int64_t)co * p.k;
    for (int j = 0; j < p.k; ++j) {
      const int ti = t0 + j * p.dil;
      if (ti >= 0 && ti < p.Tin) A += (int32_t)xr[ti] * (int32_t)wr[j];
    }
  } else {
    for (int ci = 0; ci < p.Cin; ++ci) {
      const int8_t* xr = xb + (int64_t)ci * p.Tin;
      for (int j = 0; j < p.k; ++j) {
        const int ti = t0 + j * p.dil;
        if (ti >= 0 && ti < p.Tin) {
          const int64_t wi = p.w_packed ? ((int64_t)j * p.Cout + co) * p.Cin + ci
                                        : ((int64_t)co * p.Cin + ci) * p.k + j;
          A += (int32_t)xr[ti] * (int32_t)p.w[wi];
        }
      }
    }
  }
  int32_t v = dyadic_rescale(A, p.m[co], p.s[co]);
  const int64_t o = (int64_t)b * p.ybs + (int64_t)co * p.Tout + to;
  if (p.res) v += (int32_t)p.res[o];
  p.y[o] = (int8_t)clamp_i8(v, p.relu ? 0 : -128);
}

hipError_t launch_conv_generic(const ConvParams& p, hipStream_t st) {
  const int64_t total = (int64_t)p.B * p.Cout * p.Tout;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  return launch_kernel(conv_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
}

// ------------------------------------------------------------------ weight re-ordering
__global__ __launch_bounds__(256) void pack_weights_kernel(const int8_t* __restrict__ w,
                                                          int8_t* __restrict__ wp, int Cout,
                                                          int Cin, int k) {
  const int64_t total = (int64_t)Cout * Cin * k;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // over the packed order
  if (idx >= total) return;
  const int ci = (int)(idx % Cin);
  const int co = (int)((idx / Cin) % Cout);
  const int j = (int)(idx / ((int64_t)Cin * Cout));
  wp[idx] = w[((int64_t)co * Cin + ci) * k + j];
}

hipError_t launch_pack_weights(const int8_t* w, int8_t* wp, int Cout, int Cin, int k, hipStream_t st) {
  const int64_t total = (int64_t)Cout * Cin * k;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  return launch_kernel(pack_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, st, w, wp, Cout, Cin, k);
}

}  // namespace qasr
