// A streaming probe with a chosen read : write ratio.  Not part of the method: it gives the
// benchmark a practical bandwidth ceiling for a kernel that, like the DAR hop, reads several
// times what it writes (packed partial sum + local slice in, packed partial sum out).
#include "dq_device.h"

namespace dq {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// out[j] = xor of in[j], in[j + n_out], in[j + 2 n_out], ... (16-byte words): every input word is
// read once, every output word written once, all accesses coalesced 16 bytes per lane.
__global__ __launch_bounds__(256) void k_stream(const u32x4 *__restrict__ in, size_t n_in, u32x4 *__restrict__ out,
                                                size_t n_out) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t j = (size_t)blockIdx.x * 256 + threadIdx.x; j < n_out; j += stride) {
    u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
    size_t i = j;
    for (; i + n_out < n_in; i += 2 * n_out) {  // two independent loads per round
      a ^= in[i];
      b ^= in[i + n_out];
    }
    if (i < n_in) a ^= in[i];
    out[j] = a ^ b;
  }
}

}  // namespace

hipError_t stream_probe(const void *in, size_t in_bytes, void *out, size_t out_bytes, uint32_t n_cu, hipStream_t s) {
  const size_t n_in = in_bytes / 16, n_out = out_bytes / 16;
  size_t blocks = (n_out + 255) / 256;
  const size_t resident = (size_t)n_cu * 8;
  if (blocks > resident) blocks = resident;
  hipLaunchKernelGGL(k_stream, dim3((uint32_t)blocks), dim3(256), 0, s, static_cast<const u32x4 *>(in), n_in,
                     static_cast<u32x4 *>(out), n_out);
  return hipGetLastError();
}

}  // namespace dq
