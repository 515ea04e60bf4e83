// The shallow-layer 3x3 convolution (64 -> 64 channels, weight and window resident in LDS) as a launch of its own;
// the kernel's device code and plan are in conv_rw_impl.h.
#include "conv_rw_impl.h"

namespace convbn {

using namespace rw;

namespace {

__global__ __launch_bounds__(64 * NWAVES) void conv_rw_kernel(RwParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  body(p, blockIdx.x, gridDim.x, smem);
}

hipError_t launch(const RwParams& p, hipStream_t st) {
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_rw_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL);
  });
  if (attr_err != hipSuccess) return attr_err;
  hipLaunchKernelGGL(conv_rw_kernel, dim3(ceil_div(p.M, p.L)), dim3(64 * NWAVES), LDS_TOTAL, st, p);
  return hipGetLastError();
}

}  // namespace

bool rw_fprop_supported(const Geom& g, int dtype) {
  RwParams p;
  return dtype == CONVBN_BF16 && fprop_params(g, &p);
}
bool rw_dgrad_supported(const Geom& g, int dtype) {
  RwParams p;
  return dtype == CONVBN_BF16 && dgrad_params(g, &p);
}
hipError_t launch_fprop_rw(const Geom& g, const void* x, const void* w_krsc, const float* bias, void* z,
                           hipStream_t st, const BnEpilogue* bn) {
  RwParams p;
  if (!fprop_params(g, &p)) return hipErrorInvalidValue;
  if (bn) p.bn = *bn;
  p.act = (const bf16_t*)x; p.wgt = (const bf16_t*)w_krsc; p.bias = bias; p.out = (bf16_t*)z;
  p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
  return launch(p, st);
}
hipError_t launch_dgrad_rw(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                           hipStream_t st) {
  RwParams p;
  if (!dgrad_params(g, &p)) return hipErrorInvalidValue;
  p.act = (const bf16_t*)dz; p.wgt = (const bf16_t*)w_crsk; p.bias = bias; p.out = (bf16_t*)dx;
  p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
  return launch(p, st);
}

}  // namespace convbn

#ifdef RW_TRACE
extern "C" int convbn_debug_read_rw_trace(unsigned long long* host, size_t n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(convbn::rw::rw_trace), n * sizeof(unsigned long long));
}
#endif
