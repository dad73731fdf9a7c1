// Measurement aid: the bf16 matrix-core rate the chip sustains for given operand bits.  The attention and
// calibration kernels are priced against the datasheet peak; this loop of back-to-back, independent
// v_mfma_f32_32x32x16_bf16 instructions (no memory traffic, no vector ALU work) shows what the same matrix
// pipes deliver on the machine at hand, which depends on the operand data through the power-limited clock.
#include "device_util.h"
#include "kernels.h"

namespace heatkv {

namespace {

constexpr int kProbeOperands = 4096;  // 16-byte operand slots the kernel reads (64 KB)

__global__ __launch_bounds__(256) void probe_mfma_kernel(const uint4* ops, float* out, int iters) {
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  union U {
    uint4 u;
    bf16x8 v;
  };
  U a[8], b[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j].u = ops[(threadIdx.x * 16 + j) & (kProbeOperands - 1)];
    b[j].u = ops[(threadIdx.x * 16 + 8 + j) & (kProbeOperands - 1)];
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + i) & 7].v, b[u].v, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

size_t probe_mfma_operand_bytes() { return size_t(kProbeOperands) * 16; }

hipError_t launch_probe_mfma(const void* operands, float* out, int workgroups, int iters, hipStream_t stream) {
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(256), 0, stream, static_cast<const uint4*>(operands), out,
                     iters);
  return hipGetLastError();
}

}  // namespace heatkv
