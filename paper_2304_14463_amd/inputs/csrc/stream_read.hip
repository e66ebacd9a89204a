// Measurement support: reads device arrays once with coalesced 16-byte loads and does
// nothing with them (an XOR per lane, one word written per thread at the end).  The time it
// takes over a batch of candidates is the rate at which this GPU delivers those bytes to a
// kernel at all: the attainable ceiling next to the 8 TB/s of the data sheet.  Holds no
// arithmetic of the evaluated method.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kThreads = 1024;
constexpr int kUnroll = 8;   // independent 16-byte loads in flight per lane

struct Span {
  const uint4* p;
  uint64_t n16;   // 16-byte words
};

__device__ __forceinline__ uint32_t fold(const uint4& v) { return v.x ^ v.y ^ v.z ^ v.w; }

__global__ __launch_bounds__(kThreads) void stream_read_kernel(Span a, Span b, Span c, uint32_t* __restrict__ out) {
  uint32_t acc = 0;
  const Span spans[3] = {a, b, c};
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    // every workgroup takes one contiguous stretch of the array (measured a few per cent faster
    // than striding over it with the whole grid)
    const uint4* __restrict__ p = spans[k].p;
    const uint64_t n16 = spans[k].n16;
    const uint64_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const uint64_t lo = per * blockIdx.x, hi = lo + per < n16 ? lo + per : n16;
    uint64_t i = lo + threadIdx.x;
    for (; i + (kUnroll - 1) * kThreads < hi; i += kUnroll * kThreads) {
      uint4 v[kUnroll];
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) v[j] = p[i + j * kThreads];
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) acc ^= fold(v[j]);
    }
    for (; i < hi; i += kThreads) acc ^= fold(p[i]);
  }
  out[(uint64_t)blockIdx.x * kThreads + threadIdx.x] = acc;
}

}  // namespace

// Reads bytes_x / 16 whole 16-byte words of each of the three device arrays (16-byte aligned;
// a tail of fewer than 16 bytes is left out) with `blocks` workgroups of 1024 threads and
// writes one word per thread to out (device, blocks * 1024 words).  Asynchronous on the
// stream.  Returns the hipError_t of the launch (0 = success).
extern "C" int mocgen_stream_read(const void* x0, uint64_t bytes0, const void* x1, uint64_t bytes1, const void* x2,
                                  uint64_t bytes2, int32_t blocks, uint32_t* out, void* hip_stream) {
  if (blocks <= 0 || !out) return (int)hipErrorInvalidValue;
  if (((uintptr_t)x0 | (uintptr_t)x1 | (uintptr_t)x2) & 15) return (int)hipErrorInvalidValue;
  const Span a{static_cast<const uint4*>(x0), bytes0 / 16}, b{static_cast<const uint4*>(x1), bytes1 / 16},
      c{static_cast<const uint4*>(x2), bytes2 / 16};
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                     a, b, c, out);
  return (int)hipGetLastError();
}
