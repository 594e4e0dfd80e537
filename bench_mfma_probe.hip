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


// Second aid: how many vector ALU instructions a SIMD issues for free beside its MFMAs.  Every wavefront runs the
// same loop of four independent MFMAs with a fixed group of vector instructions after each of them; the groups are
// the instruction mixes of one attention step per MFMA (v_exp, FMA, add, half a bf16 pack, with and without half a
// v_max3), and plain v_add_f32 four, five and six at a time.  Time per MFMA against the loop without vector
// instructions shows what fits under an MFMA.  Operand values do not matter (a few small integers).
#define PROBE_M(i) "v_mfma_f32_32x32x16_bf16 %[acc" #i "], %[a], %[b], %[acc" #i "]\n"
#define PROBE_FS(j) "v_fma_f32 %[x" #j "], %[sc], %[c], %[d]\n"
#define PROBE_E(j) "v_exp_f32 %[x" #j "], %[c]\n"
#define PROBE_A(j) "v_add_f32 %[x" #j "], %[x" #j "], %[c]\n"
#define PROBE_CV(j) "v_cvt_pk_bf16_f32 %[x" #j "], %[c], %[d]\n"
#define PROBE_X3(j) "v_max3_f32 %[x" #j "], %[x" #j "], %[c], %[d]\n"
#define PROBE_STEP(i, j) PROBE_FS(i) PROBE_E(i) PROBE_A(j)
#define PROBE_OPERANDS                                                                                            \
  : [acc0] "+v"(acc[0]), [acc1] "+v"(acc[1]), [acc2] "+v"(acc[2]), [acc3] "+v"(acc[3]), [x0] "+v"(x[0]),         \
    [x1] "+v"(x[1]), [x2] "+v"(x[2]), [x3] "+v"(x[3]), [x4] "+v"(x[4]), [x5] "+v"(x[5]), [x6] "+v"(x[6]),         \
    [x7] "+v"(x[7])                                                                                               \
  : [a] "v"(a), [b] "v"(b), [c] "v"(c), [d] "v"(d), [sc] "s"(sc)
#define PROBE_KERNEL(NAME, BODY)                                                                     \
  __global__ __launch_bounds__(256) void NAME(float* __restrict__ sink, int iters, float seed) {     \
    bf16x8 a, b;                                                                                     \
    for (int q = 0; q < 8; ++q) {                                                                    \
      a[q] = (__bf16)(float)((threadIdx.x + q) & 3);                                                 \
      b[q] = (__bf16)(1.0f + 0.25f * q);                                                             \
    }                                                                                                \
    f32x16 acc[4];                                                                                   \
    for (int n = 0; n < 4; ++n)                                                                      \
      for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;                                                  \
    float x[8];                                                                                      \
    for (int n = 0; n < 8; ++n) x[n] = seed + n * 0.01f;                                             \
    const float c = seed * 0.5f, d = seed * 0.25f, sc = seed * 0.125f;                               \
    for (int it = 0; it < iters; ++it) asm volatile(BODY PROBE_OPERANDS);                            \
    float s = 0.f;                                                                                   \
    for (int n = 0; n < 4; ++n)                                                                      \
      for (int r = 0; r < 16; ++r) s += acc[n][r];                                                   \
    for (int n = 0; n < 8; ++n) s += x[n];                                                           \
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;                                                \
  }
PROBE_KERNEL(overlap_none, PROBE_M(0) PROBE_M(1) PROBE_M(2) PROBE_M(3))
PROBE_KERNEL(overlap_step, PROBE_M(0) PROBE_STEP(0, 4) PROBE_CV(1) PROBE_M(1) PROBE_STEP(2, 5) PROBE_M(2)
                               PROBE_STEP(0, 6) PROBE_CV(1) PROBE_M(3) PROBE_STEP(2, 7))
PROBE_KERNEL(overlap_step_max, PROBE_M(0) PROBE_STEP(0, 4) PROBE_CV(1) PROBE_M(1) PROBE_STEP(2, 5) PROBE_X3(3)
                                   PROBE_M(2) PROBE_STEP(0, 6) PROBE_CV(1) PROBE_M(3) PROBE_STEP(2, 7) PROBE_X3(3))
PROBE_KERNEL(overlap_add4, PROBE_M(0) PROBE_A(0) PROBE_A(1) PROBE_A(2) PROBE_A(3) PROBE_M(1) PROBE_A(4) PROBE_A(5)
                               PROBE_A(6) PROBE_A(7) PROBE_M(2) PROBE_A(0) PROBE_A(1) PROBE_A(2) PROBE_A(3) PROBE_M(3)
                                   PROBE_A(4) PROBE_A(5) PROBE_A(6) PROBE_A(7))
PROBE_KERNEL(overlap_add5, PROBE_M(0) PROBE_A(0) PROBE_A(1) PROBE_A(2) PROBE_A(3) PROBE_A(4) PROBE_M(1) PROBE_A(5)
                               PROBE_A(6) PROBE_A(7) PROBE_A(0) PROBE_A(1) PROBE_M(2) PROBE_A(2) PROBE_A(3) PROBE_A(4)
                                   PROBE_A(5) PROBE_A(6) PROBE_M(3) PROBE_A(7) PROBE_A(0) PROBE_A(1) PROBE_A(2)
                                       PROBE_A(3))
PROBE_KERNEL(overlap_add6, PROBE_M(0) PROBE_A(0) PROBE_A(1) PROBE_A(2) PROBE_A(3) PROBE_A(4) PROBE_A(5) PROBE_M(1)
                               PROBE_A(6) PROBE_A(7) PROBE_A(0) PROBE_A(1) PROBE_A(2) PROBE_A(3) PROBE_M(2) PROBE_A(4)
                                   PROBE_A(5) PROBE_A(6) PROBE_A(7) PROBE_A(0) PROBE_A(1) PROBE_M(3) PROBE_A(2)
                                       PROBE_A(3) PROBE_A(4) PROBE_A(5) PROBE_A(6) PROBE_A(7))

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


// kind: 0 MFMAs only; 1 the attention step's mix per MFMA (exp, FMA, add, half a bf16 pack); 2 the same plus half a
// v_max3; 3, 4, 5: four, five, six v_add_f32 per MFMA.  Every wavefront issues 4 * iters MFMAs.
//   sink: device, >= n_workgroups * 256 floats, overwritten;  iters >= 1;  n_workgroups in [1, 65536]
// Returns 0, or -1 on bad arguments, -4 when the launch fails; only enqueues.
extern "C" int bench_valu_under_mfma(int32_t kind, float* sink, size_t sink_floats, int32_t iters,
                                     int32_t n_workgroups, void* stream) {
  if (!sink || kind < 0 || kind > 5 || iters < 1 || n_workgroups < 1 || n_workgroups > 65536) return -1;
  if (sink_floats < (size_t)n_workgroups * 256) return -1;
  typedef void (*kernel_t)(float*, int, float);
  const kernel_t table[6] = {overlap_none, overlap_step, overlap_step_max, overlap_add4, overlap_add5, overlap_add6};
  table[kind]<<<dim3(n_workgroups), 256, 0, (hipStream_t)stream>>>(sink, iters, 0.5f);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}
