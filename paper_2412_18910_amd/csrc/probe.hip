// Diagnostic: what a dependent chain of plain read-only streaming kernels sustains on this GPU.
// The decode GEMMs are such chains with arithmetic attached (every weight byte read once, one
// kernel per matrix, each launch waiting for the one before), so this is the yardstick their
// achieved GB/s is held against besides the published peak.
#include <chrono>

#include "ae_internal.h"

namespace {

// grid-stride read of n16 16-byte pieces; the xor keeps the loads alive, nothing is written
__global__ __launch_bounds__(256) void read_stream_kernel(const uint4 *src, size_t n16, uint32_t *sink) {
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const uint4 v = src[i];
    acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1u;   // never true for the zero-filled buffer
}

}  // namespace

extern "C" int ae_probe_read_stream(void *hip_stream, size_t bytes_per_launch, int launches, int repeats,
                                    double *us_per_launch) {
  if (!us_per_launch || bytes_per_launch < 4096 || bytes_per_launch % 4096 || launches < 1 || repeats < 1) return AE_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  // rotate over enough distinct buffers that no launch finds its operand in a cache (>= 1 GiB, <= 4 GiB)
  size_t nbuf = ((size_t)1 << 30) / bytes_per_launch + 1;
  if (nbuf > (size_t)launches) nbuf = launches;
  if (nbuf * bytes_per_launch > ((size_t)4 << 30)) return AE_EINVAL;
  char *buf = nullptr;
  uint32_t *sink = nullptr;
  if (hipMalloc((void **)&buf, nbuf * bytes_per_launch) != hipSuccess) return AE_ENOMEM;
  if (hipMalloc((void **)&sink, 256) != hipSuccess) { hipFree(buf); return AE_ENOMEM; }
  ae::launch_fill_zero(buf, nbuf * bytes_per_launch, s);
  ae::launch_fill_zero(sink, 256, s);
  const size_t n16 = bytes_per_launch / 16;
  auto pass = [&]() {
    for (int i = 0; i < launches; ++i)
      read_stream_kernel<<<2048, 256, 0, s>>>((const uint4 *)(buf + (size_t)(i % nbuf) * bytes_per_launch), n16, sink);
  };
  pass();
  hipError_t e = hipStreamSynchronize(s);
  const auto t0 = std::chrono::steady_clock::now();
  for (int r = 0; r < repeats && e == hipSuccess; ++r) pass();
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
  if (e == hipSuccess) e = hipGetLastError();
  hipFree(buf);
  hipFree(sink);
  if (e != hipSuccess) return AE_EHIP;
  *us_per_launch = us / ((double)repeats * launches);
  return AE_OK;
}
