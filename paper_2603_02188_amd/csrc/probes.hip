// Measurement probes of libmlra (not on the decode path): a plain streaming read, against which the decode
// kernel's achieved bandwidth can be read next to the 8 TB/s nameplate, and a shader-clock probe.
#include "mlra_internal.h"

namespace mlra {
namespace {

// Every lane reads 16 bytes per step, consecutive lanes consecutive addresses, workgroups striding over the
// buffer; the XOR of everything read goes to one dword per workgroup so that the loads cannot be dropped.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
  uint4 acc = {0u, 0u, 0u, 0u};
  const size_t stride = (size_t)gridDim.x * 256 * 4;
  for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
    // four independent loads in flight per lane
    const uint4 a = src[i];
    const uint4 b = i + 256 < n16 ? src[i + 256] : uint4{0u, 0u, 0u, 0u};
    const uint4 c = i + 512 < n16 ? src[i + 512] : uint4{0u, 0u, 0u, 0u};
    const uint4 d = i + 768 < n16 ? src[i + 768] : uint4{0u, 0u, 0u, 0u};
    acc.x ^= a.x ^ b.x ^ c.x ^ d.x;
    acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
    acc.z ^= a.z ^ b.z ^ c.z ^ d.z;
    acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
  }
  uint32_t v = acc.x ^ acc.y ^ acc.z ^ acc.w;
  for (int o = 32; o > 0; o >>= 1) v ^= __shfl_xor(v, o);
  if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], v);
}

// One wave counts shader-clock cycles against the constant 100 MHz counter for about `spin_us` microseconds.
__global__ void clock_probe_kernel(long long* out, int spin_us) {
  const long long w0 = wall_clock64(), c0 = clock64();
  long long w1 = w0;
  while (w1 - w0 < (long long)spin_us * 100) {
    __builtin_amdgcn_s_sleep(32);   // (mostly asleep: the wave shares its SIMD with whatever else runs)
    w1 = wall_clock64();
  }
  const long long c1 = clock64();
  if (threadIdx.x == 0) {
    out[0] = c1 - c0;   // shader cycles
    out[1] = w1 - w0;   // 10 ns ticks
  }
}

}  // namespace
}  // namespace mlra

using namespace mlra;

extern "C" {

int mlra_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, int32_t workgroups, void* stream) {
  if (!src || !sink) return MLRA_ERR_NULL;
  if (bytes < 16 || workgroups <= 0 || workgroups > 65536 || ((uintptr_t)src) % 16 != 0) return MLRA_ERR_SHAPE;
  stream_read_kernel<<<workgroups, 256, 0, (hipStream_t)stream>>>((const uint4*)src, bytes / 16, sink);
  return check_launch();
}

int mlra_probe_shader_clock(long long* out, int32_t spin_us, void* stream) {
  if (!out) return MLRA_ERR_NULL;
  if (spin_us <= 0 || spin_us > 100000) return MLRA_ERR_SHAPE;
  clock_probe_kernel<<<1, 64, 0, (hipStream_t)stream>>>(out, spin_us);
  return check_launch();
}

}  // extern "C"
