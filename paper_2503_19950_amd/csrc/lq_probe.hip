// Measurement helper: a plain streaming read of a device buffer.  The benchmark runs it over
// as many bytes as one decode-attention launch reads, on the same rotation of buffers, to
// report what pure reading reaches on the machine at that size (the practical ceiling the
// attention kernel is compared with, beside the nominal 8 TB/s).
#include "lq_internal.h"

namespace lq {

// Every lane reads 16 bytes per step, consecutive lanes consecutive addresses, the grid
// strides over the buffer; the xor of everything read goes to one word per workgroup so that
// the loads cannot be dropped.
__global__ void __launch_bounds__(256) read_probe_kernel(const uint4* __restrict__ p, size_t n16, uint32_t* sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {   // four loads in flight per lane
    const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const uint4 a = p[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc ^= __shfl_xor(acc, o);
  if ((threadIdx.x & 63) == 0) atomicXor(sink + blockIdx.x, acc);
}

}  // namespace lq

using namespace lq;

extern "C" lq_status logquant_read_probe(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink) return LQ_ERR_NULL;
  if (bytes < 16 || ((uintptr_t)buf & 15)) return LQ_ERR_SHAPE;
  const size_t n16 = bytes / 16;
  // two workgroups per compute unit (measured best on 57 MB .. 1.1 GB: 5.6 - 6.4 TB/s; more,
  // smaller workgroups reach 4.8 - 5.4)
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 512) blocks = 512;
  clear_stale_error();
  hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)buf, n16,
                     (uint32_t*)sink);
  return launch_status(__func__) == hipSuccess ? LQ_OK : LQ_ERR_HIP;
}
