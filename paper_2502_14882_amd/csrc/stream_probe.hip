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
// The tile quantizer's memory traffic without its arithmetic: a 256-thread block reads a tile of
// 128 tokens x 128 fp16 (32 KB, eight 16-byte loads per lane, as the quantizer does), folds it with
// a handful of instructions and writes `code_bytes` + `meta_bytes` per tile.
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) tile_traffic_kernel(const v8h* __restrict__ x,
                                                           v4u* __restrict__ codes,
                                                           float* __restrict__ meta, int code_v4,
                                                           int meta_f) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t tile = blockIdx.x;
  const v8h* src = x + (tile * 128 + 32 * wave + (lane >> 4)) * 16 + (lane & 15);
  v8h r[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = __builtin_nontemporal_load(src + (size_t)i * 64);
  v8h mn = r[0], mx = r[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) {
    mn = __builtin_elementwise_min(mn, r[i]);
    mx = __builtin_elementwise_max(mx, r[i]);
  }
  const v4u a = __builtin_bit_cast(v4u, mn), b = __builtin_bit_cast(v4u, mx);
  const v4u c = a ^ b;
  for (int i = tid; i < code_v4; i += 256) codes[tile * code_v4 + i] = c;
  const float f = __builtin_bit_cast(float, c[0] ^ c[1] ^ c[2] ^ c[3]);
  for (int i = tid; i < meta_f; i += 256) meta[tile * meta_f + i] = f;
}
}  // namespace

extern "C" int cq_bench_tile_traffic(const void* x_f16, void* codes, void* meta, size_t n_tiles,
                                     int code_bytes_per_tile, int meta_bytes_per_tile, void* stream) {
  if (!x_f16 || !codes || !meta) return CQ_ERR_NULL;
  if (((reinterpret_cast<uintptr_t>(x_f16) | reinterpret_cast<uintptr_t>(codes)) & 15u) ||
      (reinterpret_cast<uintptr_t>(meta) & 3u))
    return CQ_ERR_ALIGN;
  if (code_bytes_per_tile < 0 || code_bytes_per_tile % 16 || meta_bytes_per_tile < 0 ||
      meta_bytes_per_tile % 4 || n_tiles > 0x7fffffffu)
    return CQ_ERR_SHAPE;
  if (n_tiles == 0) return CQ_OK;
  tile_traffic_kernel<<<dim3((unsigned)n_tiles), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const v8h*>(x_f16), static_cast<v4u*>(codes), static_cast<float*>(meta),
      code_bytes_per_tile / 16, meta_bytes_per_tile / 4);
  return hipGetLastError() == hipSuccess ? CQ_OK : CQ_ERR_HIP;
}

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
