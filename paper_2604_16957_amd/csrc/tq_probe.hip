// Measurement aid, not part of the attention path: a kernel that only reads a buffer, so that the read
// bandwidth the machine delivers for a stream of a given size can be timed next to the decode kernel.
#include "tq_internal.h"

namespace tq {
namespace {
// Read-bandwidth probe: block b reads the b-th contiguous slice of the buffer, 16 bytes per lane and eight
// loads in flight per lane, non-temporal; the XOR keeps the loads alive.
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
}  // namespace

hipError_t launch_read_probe(const void* src, size_t bytes, void* sink, hipStream_t s) {
  constexpr int kBlocks = 256;
  const size_t per_block = bytes / 16 / kBlocks;          // a multiple of 8 * 512 by the caller's check
  hipLaunchKernelGGL(read_probe_kernel, dim3(kBlocks), dim3(512), 0, s, static_cast<const probe_u32x4*>(src),
                     per_block, static_cast<unsigned*>(sink));
  return hipGetLastError();
}

}  // namespace tq
