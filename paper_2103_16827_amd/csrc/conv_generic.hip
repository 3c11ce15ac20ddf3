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
          const int64_t wi = p.w_packed ? packed_weight_index(j, co, ci, p.Cout, p.Cin)
                                        : ((int64_t)co * p.Cin + ci) * p.k + j;
          A += (int32_t)xr[ti] * (int32_t)p.w[wi];
        }
      }
    }
  }
  int32_t v = dyadic_rescale(A, p.m[co], p.s[co]);
  const int64_t o = (int64_t)b * p.ybs + (int64_t)co * p.Tout + to;
  if (p.res) v += (int32_t)p.res[o];
#pragma unroll
  for (int r = 0; r < kMaxMoreRes; ++r)
    if (r < p.n_res_more) v += (int32_t)p.res_more[r][o];
  p.y[o] = (int8_t)clamp_i8(v, p.relu ? 0 : -128);
}

hipError_t launch_conv_generic(const ConvParams& p, hipStream_t st) {
  const int64_t total = (int64_t)p.B * p.Cout * p.Tout;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  return launch_kernel(conv_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
}

// ------------------------------------------------------------------ weight re-ordering
// [Cout][Cin][k] -> MFMA operand order (see packed_weight_index); one thread per packed byte.
__global__ __launch_bounds__(256) void pack_weights_kernel(const int8_t* __restrict__ w,
                                                          int8_t* __restrict__ wp, int Cout,
                                                          int Cin, int k) {
  const int co16n = (Cout + 15) >> 4, kch = Cin >> 6;
  const int64_t total = (int64_t)k * co16n * kch * 1024;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int e = (int)(idx & 15), lane = (int)((idx >> 4) & 63);
  int64_t rest = idx >> 10;
  const int kc = (int)(rest % kch);
  rest /= kch;
  const int co16 = (int)(rest % co16n);
  const int j = (int)(rest / co16n);
  const int n = lane & 15, gi = lane >> 4;
  const int co = 16 * co16 + n;
  const int ci = 64 * kc + (e < 8 ? 8 * gi + e : 32 + 8 * gi + (e - 8));
  wp[idx] = co < Cout ? w[((int64_t)co * Cin + ci) * k + j] : (int8_t)0;
}

hipError_t launch_pack_weights(const int8_t* w, int8_t* wp, int Cout, int Cin, int k, hipStream_t st) {
  const int64_t total = (int64_t)k * ((Cout + 15) / 16) * (Cin / 64) * 1024;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  return launch_kernel(pack_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, st, w, wp, Cout, Cin, k);
}

}  // namespace qasr
