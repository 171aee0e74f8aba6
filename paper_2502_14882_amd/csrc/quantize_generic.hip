// Shape-agnostic quantizer kernels: any head_dim (multiple of 32), any group, b in {1,2,4,8}.
//
// They evaluate the quantize equation of Sec. 2.2 element by element in fp64, where every
// intermediate is exact (fp16 inputs are multiples of 2^-24 below 2^16, so x-min, max-min and
// their products with 2^b-1 <= 255 fit 53 bits); the single rounding is the fp64 division, whose
// quotient is further from a half-integer than its rounding error unless it is an exact tie,
// so round-to-nearest-even of it equals exact rational rounding with ties to even.
// The tuned kernels replace this by per-group fp16 thresholds; these stay as the reference
// path for every other shape.
#include <hip/hip_fp16.h>

#include "cq_internal.h"

namespace cq {
namespace {

constexpr int kTileTokens = 32;
constexpr int kMaxDim = 256;

__device__ inline uint16_t canonical_min_bits(float mn) {
  uint16_t bits = __half_as_ushort(__float2half_rn(mn));  // exact: mn is an fp16 value
  return (bits & 0x7fffu) == 0 ? (uint16_t)0 : bits;      // a zero minimum is stored as +0
}

__device__ inline uint32_t exact_code(float x, double alpha, double D, double L) {
  if (!(D > 0.0)) return 0u;
  return (uint32_t)rint(((double)x - alpha) * L / D);
}

// One block per (row, token group); one thread per channel.
__global__ void quantize_channel_axis(const __half* __restrict__ x, uint32_t* __restrict__ codes,
                                      float* __restrict__ scale, uint16_t* __restrict__ minv,
                                      int n_vis, int d, int bits, int group) {
  __shared__ uint8_t tile[kTileTokens][kMaxDim];
  const int n_groups = n_vis / group;
  const size_t blk = blockIdx.x;
  const size_t row = blk / n_groups;
  const int t = (int)(blk % n_groups);
  const int c = threadIdx.x;
  const size_t tok0 = row * (size_t)n_vis + (size_t)t * group;
  const __half* xg = x + tok0 * d;

  float mn = __half2float(xg[c]), mx = mn;
  for (int j = 1; j < group; ++j) {
    const float v = __half2float(xg[(size_t)j * d + c]);
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  }
  const uint16_t mbits = canonical_min_bits(mn);
  const double alpha = (double)__half2float(__ushort_as_half(mbits));
  const double L = (double)((1 << bits) - 1);
  const double D = ((double)mx - alpha) + 0.0;  // "+ 0.0": a zero range is +0, so is its scale
  const size_t meta = (row * n_groups + t) * (size_t)d + c;
  scale[meta] = (float)(D / L);
  minv[meta] = mbits;

  const int wpt = d * bits / 32, per = 32 / bits;
  for (int j0 = 0; j0 < group; j0 += kTileTokens) {
    const int nt = min(kTileTokens, group - j0);
    for (int j = 0; j < nt; ++j)
      tile[j][c] = (uint8_t)exact_code(__half2float(xg[(size_t)(j0 + j) * d + c]), alpha, D, L);
    __syncthreads();
    for (int idx = c; idx < nt * wpt; idx += d) {
      const int j = idx / wpt, w = idx % wpt;
      uint32_t word = 0;
      for (int i = 0; i < per; ++i) word |= (uint32_t)tile[j][w * per + i] << (32 - bits * (1 + i));
      codes[(tok0 + j0 + j) * wpt + w] = word;
    }
    __syncthreads();
  }
}

// One thread per (token, channel group).
__global__ void quantize_token_axis(const __half* __restrict__ x, uint32_t* __restrict__ codes,
                                    float* __restrict__ scale, uint16_t* __restrict__ minv,
                                    size_t n_tokens, int d, int bits, int group) {
  const int ng = d / group;
  const size_t item = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (item >= n_tokens * ng) return;
  const size_t tok = item / ng;
  const int cg = (int)(item % ng);
  const __half* p = x + tok * d + (size_t)cg * group;
  float mn = __half2float(p[0]), mx = mn;
  for (int i = 1; i < group; ++i) {
    const float v = __half2float(p[i]);
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  }
  const uint16_t mbits = canonical_min_bits(mn);
  const double alpha = (double)__half2float(__ushort_as_half(mbits));
  const double L = (double)((1 << bits) - 1);
  const double D = ((double)mx - alpha) + 0.0;  // "+ 0.0": a zero range is +0, so is its scale
  scale[item] = (float)(D / L);
  minv[item] = mbits;
  const int wpt = d * bits / 32, per = 32 / bits, wpg = group * bits / 32;
  uint32_t* out = codes + tok * wpt + (size_t)cg * wpg;
  for (int w = 0; w < wpg; ++w) {
    uint32_t word = 0;
    for (int i = 0; i < per; ++i)
      word |= exact_code(__half2float(p[w * per + i]), alpha, D, L) << (32 - bits * (1 + i));
    out[w] = word;
  }
}

}  // namespace

hipError_t launch_quantize_generic(const void* x_f16, const cq_qtensor_t& out, int rows, int n_vis,
                                   int d, int bits, int axis, int group, hipStream_t stream) {
  const __half* x = static_cast<const __half*>(x_f16);
  if (axis == CQ_AXIS_CHANNEL) {
    const size_t blocks = (size_t)rows * (size_t)(n_vis / group);
    if (blocks > 0x7fffffffu) return hipErrorInvalidConfiguration;
    quantize_channel_axis<<<dim3((unsigned)blocks), dim3(d), 0, stream>>>(
        x, out.codes, out.scale, out.min, n_vis, d, bits, group);
  } else {
    const size_t n_tokens = (size_t)rows * (size_t)n_vis;
    const size_t items = n_tokens * (size_t)(d / group);
    const size_t blocks = (items + 255) / 256;
    if (blocks > 0x7fffffffu) return hipErrorInvalidConfiguration;
    quantize_token_axis<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
        x, out.codes, out.scale, out.min, n_tokens, d, bits, group);
  }
  return hipGetLastError();
}

}  // namespace cq
