// Two machine probes for the benchmark: what a plain streaming read and a register-resident
// bf16 MFMA loop reach on the GPU at hand, so that a kernel's fraction of the published
// peaks (8 TB/s, 2.5 PFLOP/s) can be read beside its fraction of what the machine gives.
// Neither is part of the attention path.
#include "lra_attn_measure.h"
#include "lra_common.h"

namespace lra {

typedef __bf16 pr_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pr_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int pr_u32x4 __attribute__((ext_vector_type(4)));

// Every thread reads 16-byte pieces a whole grid apart (consecutive lanes read consecutive
// pieces), eight requests in flight per pass; the xor of everything read goes to sink so that
// no load can be dropped.
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const pr_u32x4* __restrict__ src, size_t n16, uint32_t* sink) {
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    pr_u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const pr_u32x4 v = __builtin_nontemporal_load(src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;  // practically never: the store only keeps the loads alive
}

// Four independent 32x32 accumulators per wave, operands in registers, no memory traffic:
// iters x 4 v_mfma_f32_32x32x16_bf16 per wave (32768 flop each).  RANDOM = false: two smooth
// operand values, the same for every product; RANDOM = true: four operand registers of
// pseudo-random bf16 values in [-1, 1) taken in rotation, so that consecutive products see
// unrelated bits, as the products of a real kernel do (the clock under matrix load depends on it).
template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(int iters, float* sink) {
  const float seed = static_cast<float>(threadIdx.x & 7) * 0.125f;
  pr_bf16x8 a, b, a2, b2;
  uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if (RANDOM) {
      float v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        h = h * 1664525u + 1013904223u;
        v[k] = static_cast<float>(static_cast<int>(h >> 8) - (1 << 23)) * (1.0f / (1 << 23));
      }
      a[e] = static_cast<__bf16>(v[0]);
      b[e] = static_cast<__bf16>(v[1]);
      a2[e] = static_cast<__bf16>(v[2]);
      b2[e] = static_cast<__bf16>(v[3]);
    } else {
      a[e] = a2[e] = static_cast<__bf16>(seed + e * 0.015625f);
      b[e] = b2[e] = static_cast<__bf16>(0.5f - seed);
    }
  }
  pr_f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int e = 0; e < 16; ++e) c0[e] = c1[e] = c2[e] = c3[e] = 0.f;
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b2, a2, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, a, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, b2, c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 16; ++e) s += c0[e] + c1[e] + c2[e] + c3[e];
  if (s == 12345.678f) sink[0] = s;  // keeps the accumulators alive
}

}  // namespace lra

using namespace lra;

extern "C" {

lra_status lra_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return LRA_ERR_NULL;
  if (bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15)) return LRA_ERR_SHAPE;
  // sixteen workgroups of four waves per CU: enough requests in flight to cover the memory latency
  hipLaunchKernelGGL(probe_stream_read_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const pr_u32x4*>(src), bytes / 16, static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? LRA_OK : LRA_ERR_HIP;
}

lra_status lra_probe_mfma_bf16(int32_t iters, int32_t random_operands, int64_t* flops, void* sink, void* stream) {
  if (!sink) return LRA_ERR_NULL;
  if (iters < 1 || iters > (1 << 24)) return LRA_ERR_SHAPE;
  constexpr int kGroups = 256 * 2;  // two workgroups of four waves per CU: two waves per SIMD
  if (random_operands)
    hipLaunchKernelGGL(probe_mfma_bf16_kernel<true>, dim3(kGroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters,
                       static_cast<float*>(sink));
  else
    hipLaunchKernelGGL(probe_mfma_bf16_kernel<false>, dim3(kGroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters,
                       static_cast<float*>(sink));
  if (flops) *flops = static_cast<int64_t>(kGroups) * 4 /*waves*/ * 4 /*accumulators*/ * iters * (2LL * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? LRA_OK : LRA_ERR_HIP;
}

}  // extern "C"
