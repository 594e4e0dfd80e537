// Measurement aid of bench.py, not part of the library or of the method: a resident loop of
// independent bf16 MFMAs on operands the caller supplies.  With random operands it shows what the
// matrix cores of this part sustain under their power limit, the second denominator bench.py prints
// beside the nominal peak.  Built into its own shared object (bench_mfma_probe.so) next to bench.py.
//
//   operands_bf16 : device, >= 65,536 bytes of bf16 values, 16-byte aligned, read only
//   sink          : device, >= n_workgroups * 256 floats, overwritten
//   iters         : even, >= 2;  n_workgroups in [1, 65536]
// Runs n_workgroups x 4 wavefronts, each issuing 4 * iters independent v_mfma_f32_32x32x16_bf16
// (32,768 FLOP each).  Returns 0, or -1 on bad arguments, -4 when the launch fails; only enqueues.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_probe_kernel(const u32x4* __restrict__ operands, float* __restrict__ sink,
                                                         int iters) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    a[n] = __builtin_bit_cast(bf16x8, operands[(threadIdx.x * 8 + n) & 4095]);
    b[n] = __builtin_bit_cast(bf16x8, operands[(threadIdx.x * 8 + 4 + n + blockIdx.x) & 4095]);
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; it += 2) {   // 8 MFMAs on 4 independent accumulators per pass
#pragma unroll
    for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n], b[n], acc[n], 0, 0, 0);
#pragma unroll
    for (int n = 0; n < 4; ++n)
      acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(n + 1) & 3], b[(n + 2) & 3], acc[n], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

extern "C" int bench_mfma_probe(const void* operands_bf16, size_t operand_bytes, float* sink, size_t sink_floats,
                                int32_t iters, int32_t n_workgroups, void* stream) {
  if (!operands_bf16 || !sink) return -1;
  if (iters < 2 || (iters & 1) || n_workgroups < 1 || n_workgroups > 65536) return -1;
  if (operand_bytes < 65536 || sink_floats < (size_t)n_workgroups * 256) return -1;
  if (((uintptr_t)operands_bf16 & 15u) != 0) return -1;
  mfma_probe_kernel<<<dim3(n_workgroups), 256, 0, (hipStream_t)stream>>>((const u32x4*)operands_bf16, sink, iters);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}
