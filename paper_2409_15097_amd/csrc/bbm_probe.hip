// Hardware-ceiling probe of libbbm: a kernel that issues nothing but bf16 matrix instructions, so that the rate the
// attention kernels reach can be set against what the chip sustains on the same kind of operands.  Not part of the
// method; bench.py times it with events of its own.
#include "bbm_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeGroups = 256, kProbeThreads = 256, kProbeChain = 16;

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
// Sum of four uniform 16-bit draws, centred and scaled to unit variance: close enough to normal for a power probe.
__device__ __forceinline__ float near_normal(uint32_t seed) {
  const uint32_t h = mix32(seed), g = mix32(h + 12345u);
  return (((h & 0xffff) + (h >> 16) + (g & 0xffff) + (g >> 16)) * (1.0f / 65536.0f) - 2.0f) * 1.7320508f;
}

// One wave per SIMD; eight A and eight B fragments per lane stay in registers, four accumulators take turns, so the
// matrix pipe never waits.  RANDOM = false: every operand element is the same small constant.
template <bool RANDOM>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(float* sink, long iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int f = 0; f < 8; ++f)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t s = threadIdx.x * 977u + blockIdx.x * 131071u + f * 17u + e;
      a[f][e] = (__bf16)(RANDOM ? near_normal(s) : 1.0f);
      b[f][e] = (__bf16)(RANDOM ? near_normal(s + 77777u) : 0.5f);
    }
  f32x16 c[4] = {{0}, {0}, {0}, {0}};
  for (long it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < kProbeChain; ++n)
      c[n & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n & 7], b[(n + (n >> 3)) & 7], c[n & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += c[q][e];
  sink[blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace

extern "C" __attribute__((visibility("default"))) int bbm_probe_mfma_bf16(int normal_operands, int64_t iters, float* sink, void* stream) {
  using namespace bbm;
  clear_error();
  if (!sink) return fail(BBM_EINVAL, "bbm_probe_mfma_bf16: sink must not be NULL");
  if (iters < 1 || iters > (1ll << 24)) return fail(BBM_EINVAL, "bbm_probe_mfma_bf16: iters=%lld outside [1, 2^24]", (long long)iters);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (normal_operands) mfma_probe_kernel<true><<<kProbeGroups, kProbeThreads, 0, st>>>(sink, (long)iters);
  else mfma_probe_kernel<false><<<kProbeGroups, kProbeThreads, 0, st>>>(sink, (long)iters);
  return launch_status("bbm_probe_mfma_bf16");
}

extern "C" __attribute__((visibility("default"))) double bbm_probe_mfma_bf16_flop(int64_t iters) {
  // 256 work-groups x 4 waves x iters x 16 instructions x (32 x 32 x 16 multiply-adds = 32768 flop)
  return iters < 1 ? 0.0 : (double)kProbeGroups * (kProbeThreads / 64) * (double)iters * kProbeChain * 32768.0;
}
