// Measurement aid of bench.py, not part of the attention library: a kernel that only reads a buffer, so that the
// read bandwidth the machine delivers for a read-once stream of a given size can be timed next to the decode
// kernel (the ceiling its roofline fraction can be read against).  Built into libbench_probe.so beside bench.py.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {
// Block b reads the b-th contiguous slice of the buffer, 16 bytes per lane and eight loads in flight per lane,
// non-temporal (the policy the decode kernel streams the cache with); the XOR keeps the loads alive.
typedef uint32_t probe_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(512) void read_probe_kernel(const probe_u32x4* __restrict__ src, size_t per_block,
                                                         unsigned* sink) {
  const probe_u32x4* p = src + (size_t)blockIdx.x * per_block;
  probe_u32x4 acc = {0, 0, 0, 0};
  for (size_t i = threadIdx.x; i + 7 * 512 < per_block; i += 8 * 512) {
    probe_u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 512);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x5EEDF00Du) *sink = 1;
}
constexpr int kBlocks = 256;
}  // namespace

// Reads `bytes` (a multiple of 16 MiB) of device memory at `src` (16-byte aligned) once, 256 blocks each reading
// one contiguous slice, and does nothing else (a 4-byte result goes to `sink`, device memory, only if the XOR of
// all words equals a magic value).  Returns 0, or -1 for bad arguments, -2 if the launch failed.
extern "C" int bench_probe_read_stream(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(sink) & 3)) return -1;
  if (bytes == 0 || bytes % ((size_t)kBlocks * 8 * 512 * 16) != 0) return -1;   // whole unrolled rounds of every block
  const size_t per_block = bytes / 16 / kBlocks;
  hipLaunchKernelGGL(read_probe_kernel, dim3(kBlocks), dim3(512), 0, static_cast<hipStream_t>(stream),
                     static_cast<const probe_u32x4*>(src), per_block, static_cast<unsigned*>(sink));
  return hipGetLastError() == hipSuccess ? 0 : -2;
}
