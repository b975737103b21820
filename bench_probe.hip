// Measurement aid of bench.py, not part of the KV-cache library: built into libbench_probe.so
// beside this file (bench_probe.py).
// Calibration kernel for the attention roofline: the rate at which this GPU issues the MFMA
// instruction the attention kernel is built on (v_mfma_f32_32x32x16 with 2-byte operands),
// with nothing else going on, on operand values supplied by the caller.  The rate depends on
// those values: the matrix pipes draw more power the more operand bits change from one
// instruction to the next, and the clock follows.  Constant operands show the nominal rate;
// operands drawn like the workload's show what a kernel working on such data can reach.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 256;   // 4 wavefronts: one per SIMD
constexpr int kFrags = 8;            // distinct A and B operand fragments in rotation
constexpr int kChains = 4;           // independent accumulators

template <typename V> struct Issue;
template <> struct Issue<f16x8> {
  static __device__ __forceinline__ f32x16 run(f16x8 a, f16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};
template <> struct Issue<bf16x8> {
  static __device__ __forceinline__ f32x16 run(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};

// Every lane loads kFrags A and kFrags B fragments (16 bytes each) from `operands` and then
// issues iters x 64 MFMAs over them, fragment (j % 8) of each per instruction.
template <typename V>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(const u32x4* operands,
                                                                   int iters, float* sink) {
  V a[kFrags], b[kFrags];
  const int lane_id = blockIdx.x % 16 * kProbeThreads + threadIdx.x;   // 16 blocks' worth of data
#pragma unroll
  for (int i = 0; i < kFrags; ++i) {
    a[i] = __builtin_bit_cast(V, operands[(2 * i) * 16 * kProbeThreads + lane_id]);
    b[i] = __builtin_bit_cast(V, operands[(2 * i + 1) * 16 * kProbeThreads + lane_id]);
  }
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 64; ++j)
      acc[j % kChains] = Issue<V>::run(a[j % kFrags], b[(j / kFrags) % kFrags], acc[j % kChains]);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace

extern "C" {

// bytes of operand values a launch reads
size_t bench_mfma_probe_operand_bytes(void) {
  return (size_t)2 * kFrags * 16 * kProbeThreads * sizeof(u32x4);   // 1 MiB
}

// Launches `blocks` workgroups of 4 wavefronts that each issue iters x 64 MFMAs on fragments read
// from `operands` (device, bench_mfma_probe_operand_bytes() bytes of 2-byte values: dtype 0 =
// fp16, 1 = bf16).  sink: device, blocks x 256 floats, overwritten.  *flops_out (host, may be
// NULL): floating-point operations issued.  Asynchronous on `stream`; the caller times it.
// Returns 0, or 1 on bad arguments, 2 if the launch failed.
int32_t bench_mfma_probe(int32_t dtype, const void* operands, int32_t blocks, int32_t iters,
                         float* sink, int64_t* flops_out, void* stream) {
  if (!operands || !sink || (reinterpret_cast<uintptr_t>(operands) & 15u) || blocks <= 0 ||
      iters <= 0 || (dtype != 0 && dtype != 1))
    return 1;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const u32x4* ops = static_cast<const u32x4*>(operands);
  if (dtype == 0)
    hipLaunchKernelGGL(mfma_probe_kernel<f16x8>, dim3(blocks), dim3(kProbeThreads), 0, hs, ops,
                       iters, sink);
  else
    hipLaunchKernelGGL(mfma_probe_kernel<bf16x8>, dim3(blocks), dim3(kProbeThreads), 0, hs, ops,
                       iters, sink);
  if (flops_out)   // 32 x 32 x 16 multiply-adds per instruction
    *flops_out = (int64_t)blocks * (kProbeThreads / 64) * iters * 64 * (2ll * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

}  // extern "C"
