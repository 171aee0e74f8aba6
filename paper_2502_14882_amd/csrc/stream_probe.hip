// Measurement aid: a plain streaming read of a device buffer, the practical ceiling that the
// roofline fractions of the method's kernels are compared with.  Not part of the method.
#include "cq_internal.h"

namespace {
typedef float v4f __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256) stream_read_kernel(const v4f* __restrict__ in, size_t n4,
                                                          float* sink) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  v4f acc = {0.f, 0.f, 0.f, 0.f};
  // two non-temporal 16-byte loads in flight per lane: the fastest of the variants tried
  // (more unrolling and more blocks were slower on this chip)
  for (; i + stride < n4; i += 2 * stride) {
    const v4f a = __builtin_nontemporal_load(in + i), b = __builtin_nontemporal_load(in + i + stride);
    acc += a + b;
  }
  for (; i < n4; i += stride) acc += __builtin_nontemporal_load(in + i);
  const float s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  if (s == 1.2345e-30f && sink) *sink = s;      // keeps the loads alive, practically never true
}
__global__ void __launch_bounds__(256) stream_copy_kernel(const v4f* __restrict__ in,
                                                          v4f* __restrict__ out, size_t n4) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n4; i += stride) out[i] = in[i];
}
}  // namespace

extern "C" int cq_bench_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u))
    return CQ_ERR_NULL;
  const size_t n4 = bytes / 16;
  if (n4 == 0) return CQ_OK;
  stream_copy_kernel<<<dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const v4f*>(src), static_cast<v4f*>(dst), n4);
  return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

extern "C" int cq_bench_stream_read(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || (reinterpret_cast<uintptr_t>(buf) & 15u) != 0) return CQ_ERR_NULL;
  const size_t n4 = bytes / 16;
  if (n4 == 0) return CQ_OK;
  stream_read_kernel<<<dim3(256 * 4), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const v4f*>(buf), n4, static_cast<float*>(sink));
  return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}
