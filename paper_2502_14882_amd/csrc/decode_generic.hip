// Shape-agnostic decode attention over the packed cache: three plain kernels.
//
//   scores   raw logits s = softmax_scale * q . k_deq (visual, from packed codes) and
//            softmax_scale * q . k_text (text tail) into the workspace, with the min and max of
//            every chunk of tokens (Sec. 2.1 logits on the dequantized keys of Sec. 3.2)
//   pv       per chunk: calibrate the visual logits with g of Sec. 3.2 (gamma, delta reduced from
//            the chunk extrema), p = exp(s' - m_chunk), l = sum p, acc = sum p * v_deq
//   combine  merge the chunk partials of the joint softmax and round to fp16
//
// Works for every layout the ABI accepts (any head_dim, group, axis, b in {1,2,4,8}) by
// dequantizing element by element (code * scale + min, Sec. 2.2).  The tuned kernels are the fast
// path; this one is the fallback and the on-device cross-check.
#include <hip/hip_fp16.h>

#include <cfloat>

#include "cq_internal.h"

namespace cq {
namespace {

constexpr int kHeadBlock = 8;   // query heads of one KV head handled per pass
constexpr int kMaxDim = 256;
constexpr int kScoreThreads = 256;
constexpr int kPvTile = 64;

struct QParams {   // one quantized tensor as the kernels see it
  const uint32_t* codes;
  const float* scale;
  const uint16_t* minv;
  int axis, group;
};

__device__ inline float dequant(const QParams& t, size_t row, int n_vis, int d, int bits, int j,
                                int c, uint32_t word) {
  const int per = 32 / bits;
  const uint32_t code = (word >> (32 - bits * (1 + (c % per)))) & ((1u << bits) - 1u);
  size_t meta;
  if (t.axis == CQ_AXIS_CHANNEL)
    meta = (row * (size_t)(n_vis / t.group) + (size_t)(j / t.group)) * d + c;
  else
    meta = (row * (size_t)n_vis + j) * (size_t)(d / t.group) + c / t.group;
  return (float)code * t.scale[meta] + __half2float(__ushort_as_half(t.minv[meta]));
}

// grid.x = rows * n_chunks.  Thread per token of the chunk.
__global__ void __launch_bounds__(kScoreThreads)
scores_kernel(DecodeShape s, const __half* __restrict__ q, QParams k,
              const __half* __restrict__ k_text, const int32_t* __restrict__ n_text_dev,
              float softmax_scale, float* __restrict__ logits, float* __restrict__ minmax) {
  __shared__ float qs[kHeadBlock][kMaxDim];
  __shared__ float red_min[kScoreThreads], red_max[kScoreThreads];
  // rows of the logit array are laid out for the host's bound of the tail length; a length held
  // in device memory only shortens what is computed (chunks past it stay empty)
  const int n_all = s.n_vis + s.n_text;
  if (n_text_dev) s.n_text = min(max(*n_text_dev, 0), s.n_text);
  const int chunk = blockIdx.x % s.n_chunks;
  const size_t row = blockIdx.x / s.n_chunks;   // b * Hkv + kvh
  const int b = (int)(row / s.Hkv), kvh = (int)(row % s.Hkv);
  const bool is_text = chunk >= s.n_vis_chunks;
  const int j0 = is_text ? (chunk - s.n_vis_chunks) * kTextChunk : chunk * kVisChunk;
  const int j1 = is_text ? min(j0 + kTextChunk, s.n_text) : min(j0 + kVisChunk, s.n_vis);
  const int per = 32 / s.bits;

  for (int hb = 0; hb < s.g; hb += kHeadBlock) {
    const int nh = min(kHeadBlock, s.g - hb);
    __syncthreads();
    for (int i = threadIdx.x; i < nh * s.d; i += blockDim.x) {
      const int h = i / s.d, c = i % s.d;
      qs[h][c] = __half2float(q[((size_t)b * s.Hq + (size_t)kvh * s.g + hb + h) * s.d + c]);
    }
    __syncthreads();
    float mn[kHeadBlock], mx[kHeadBlock];
    for (int h = 0; h < kHeadBlock; ++h) { mn[h] = FLT_MAX; mx[h] = -FLT_MAX; }
    for (int j = j0 + threadIdx.x; j < j1; j += blockDim.x) {
      float acc[kHeadBlock];
      for (int h = 0; h < kHeadBlock; ++h) acc[h] = 0.f;
      if (is_text) {
        const __half* kt = k_text + (row * (size_t)s.n_text_cap + j) * s.d;
        for (int c = 0; c < s.d; ++c) {
          const float kv = __half2float(kt[c]);
          for (int h = 0; h < nh; ++h) acc[h] += qs[h][c] * kv;
        }
      } else {
        const uint32_t* cw = k.codes + (row * (size_t)s.n_vis + j) * s.words_per_token;
        uint32_t word = 0;
        for (int c = 0; c < s.d; ++c) {
          if (c % per == 0) word = cw[c / per];
          const float kv = dequant(k, row, s.n_vis, s.d, s.bits, j, c, word);
          for (int h = 0; h < nh; ++h) acc[h] += qs[h][c] * kv;
        }
      }
      for (int h = 0; h < nh; ++h) {
        const float v = acc[h] * softmax_scale;
        const size_t hq = (size_t)b * s.Hq + (size_t)kvh * s.g + hb + h;
        logits[hq * n_all + (is_text ? s.n_vis + j : j)] = v;
        mn[h] = fminf(mn[h], v);
        mx[h] = fmaxf(mx[h], v);
      }
    }
    for (int h = 0; h < nh; ++h) {
      __syncthreads();
      red_min[threadIdx.x] = mn[h];
      red_max[threadIdx.x] = mx[h];
      __syncthreads();
      for (int off = blockDim.x / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) {
          red_min[threadIdx.x] = fminf(red_min[threadIdx.x], red_min[threadIdx.x + off]);
          red_max[threadIdx.x] = fmaxf(red_max[threadIdx.x], red_max[threadIdx.x + off]);
        }
        __syncthreads();
      }
      if (threadIdx.x == 0) {
        const size_t hq = (size_t)b * s.Hq + (size_t)kvh * s.g + hb + h;
        minmax[(hq * s.n_chunks + chunk) * 2 + 0] = red_min[0];
        minmax[(hq * s.n_chunks + chunk) * 2 + 1] = red_max[0];
      }
    }
  }
}

// grid.x = rows * n_chunks.  Thread per output channel.
__global__ void pv_kernel(DecodeShape s, QParams v, const __half* __restrict__ v_text,
                          const int32_t* __restrict__ n_text_dev, Calib cal,
                          const float* __restrict__ logits, const float* __restrict__ minmax,
                          float* __restrict__ partial) {
  __shared__ float p[kHeadBlock][kPvTile];
  __shared__ float slope_s[kHeadBlock], gamma_s[kHeadBlock], shift_s[kHeadBlock], m_s[kHeadBlock];
  const int n_all = s.n_vis + s.n_text;       // row pitch of the logits: the host's bound
  if (n_text_dev) s.n_text = min(max(*n_text_dev, 0), s.n_text);
  const int chunk = blockIdx.x % s.n_chunks;
  const size_t row = blockIdx.x / s.n_chunks;
  const int b = (int)(row / s.Hkv), kvh = (int)(row % s.Hkv);
  const bool is_text = chunk >= s.n_vis_chunks;
  const int j0 = is_text ? (chunk - s.n_vis_chunks) * kTextChunk : chunk * kVisChunk;
  const int j1 = is_text ? min(j0 + kTextChunk, s.n_text) : min(j0 + kVisChunk, s.n_vis);
  const int c = threadIdx.x;
  const int per = 32 / s.bits;

  for (int hb = 0; hb < s.g; hb += kHeadBlock) {
    const int nh = min(kHeadBlock, s.g - hb);
    __syncthreads();
    if (c < nh) {
      const size_t hq = (size_t)b * s.Hq + (size_t)kvh * s.g + hb + c;
      const float* mm = minmax + hq * s.n_chunks * 2;
      float slope = 1.f, gamma = 0.f, shift = 0.f;   // s' = slope * (s - gamma) + shift
      if (!is_text && cal.mode != CQ_CALIB_NONE) {
        float lo = cal.gamma, hi = cal.delta;
        if (cal.mode == CQ_CALIB_DYNAMIC) {
          lo = FLT_MAX; hi = -FLT_MAX;
          for (int i = 0; i < s.n_vis_chunks; ++i) {
            lo = fminf(lo, mm[2 * i]);
            hi = fmaxf(hi, mm[2 * i + 1]);
          }
        }
        const float width = hi - lo;
        slope = width == 0.f ? 1.f : (width + cal.tau1 - cal.tau2) / width;
        gamma = lo;
        shift = lo - cal.tau1;
      }
      const float clo = slope * (mm[2 * chunk] - gamma) + shift;
      const float chi = slope * (mm[2 * chunk + 1] - gamma) + shift;
      slope_s[c] = slope; gamma_s[c] = gamma; shift_s[c] = shift;
      // the map is monotone, so an end point is the chunk maximum; a chunk without tokens (beyond
      // a tail length read from device memory) must not set the reference point of the combine
      m_s[c] = j1 > j0 ? fmaxf(clo, chi) : -FLT_MAX;
    }
    __syncthreads();
    float acc[kHeadBlock], l[kHeadBlock];
    for (int h = 0; h < kHeadBlock; ++h) { acc[h] = 0.f; l[h] = 0.f; }
    for (int t0 = j0; t0 < j1; t0 += kPvTile) {
      const int nt = min(kPvTile, j1 - t0);
      __syncthreads();
      for (int i = c; i < nh * nt; i += blockDim.x) {
        const int h = i / nt, jj = i % nt;
        const size_t hq = (size_t)b * s.Hq + (size_t)kvh * s.g + hb + h;
        const float raw = logits[hq * n_all + (is_text ? s.n_vis : 0) + t0 + jj];
        p[h][jj] = expf(slope_s[h] * (raw - gamma_s[h]) + shift_s[h] - m_s[h]);
      }
      __syncthreads();
      for (int jj = 0; jj < nt; ++jj) {
        const int j = t0 + jj;
        float val;
        if (is_text) {
          val = __half2float(v_text[(row * (size_t)s.n_text_cap + j) * s.d + c]);
        } else {
          const uint32_t word = v.codes[(row * (size_t)s.n_vis + j) * s.words_per_token + c / per];
          val = dequant(v, row, s.n_vis, s.d, s.bits, j, c, word);
        }
        for (int h = 0; h < nh; ++h) {
          acc[h] += p[h][jj] * val;
          l[h] += p[h][jj];
        }
      }
    }
    for (int h = 0; h < nh; ++h) {
      const size_t hq = (size_t)b * s.Hq + (size_t)kvh * s.g + hb + h;
      float* out = partial + (hq * s.n_chunks + chunk) * (size_t)(s.d + 2);
      if (c == 0) { out[0] = m_s[h]; out[1] = l[h]; }
      out[2 + c] = acc[h];
    }
  }
}

// grid.x = B * Hq.  Thread per output channel.
__global__ void combine_kernel(int n_chunks, int d, const float* __restrict__ partial,
                               __half* __restrict__ out) {
  const size_t hq = blockIdx.x;
  const int c = threadIdx.x;
  const float* base = partial + hq * n_chunks * (size_t)(d + 2);
  // Sixteen chunks at a time, all of their loads independent of each other and of the running
  // sums: with up to 16 chunks a thread waits for memory once.  Each batch brings its own
  // reference point; the sums so far are rescaled when it is larger (online softmax over batches).
  // A chunk without tokens has m = -FLT_MAX and weight 0.
  float M = -FLT_MAX, num = 0.f, den = 0.f;
  for (int i0 = 0; i0 < n_chunks; i0 += 16) {
    float m[16], l[16], acc[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const float* pi = base + (size_t)min(i0 + u, n_chunks - 1) * (d + 2);
      m[u] = pi[0];
      l[u] = pi[1];
      acc[u] = pi[2 + c];
    }
    float Mb = M;
#pragma unroll
    for (int u = 0; u < 16; ++u) Mb = fmaxf(Mb, m[u]);       // a repeated (clamped) chunk changes nothing
    const float keep = expf(M - Mb);                          // 1 when the reference stays, 0 at the start
    num *= keep;
    den *= keep;
    M = Mb;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const float w = i0 + u < n_chunks ? expf(m[u] - M) : 0.f;
      num = fmaf(w, acc[u], num);
      den = fmaf(w, l[u], den);
    }
  }
  out[hq * d + c] = __float2half_rn(num / den);
}

}  // namespace

hipError_t launch_combine(int n_rows, int n_chunks, int d, const float* partial, void* out,
                          hipStream_t stream) {
  combine_kernel<<<dim3((unsigned)n_rows), dim3(d), 0, stream>>>(n_chunks, d, partial,
                                                                 static_cast<__half*>(out));
  return hipGetLastError();
}

hipError_t launch_scores_generic(const DecodeShape& s, const void* q, const cq_qtensor_t& k,
                                 const void* k_text, const int32_t* n_text_dev,
                                 float softmax_scale, float* logits, float* minmax,
                                 hipStream_t stream) {
  const size_t blocks = (size_t)s.B * s.Hkv * (size_t)s.n_chunks;
  if (blocks > 0x7fffffffu) return hipErrorInvalidConfiguration;
  QParams kp{k.codes, k.scale, k.min, s.k_axis, s.k_group};
  scores_kernel<<<dim3((unsigned)blocks), dim3(kScoreThreads), 0, stream>>>(
      s, static_cast<const __half*>(q), kp, static_cast<const __half*>(k_text), n_text_dev,
      softmax_scale, logits, minmax);
  return hipGetLastError();
}

hipError_t launch_decode_generic(const DecodeShape& s, const void* q, const cq_qtensor_t& k,
                                 const cq_qtensor_t& v, const void* k_text, const void* v_text,
                                 const int32_t* n_text_dev, const Calib& calib,
                                 float softmax_scale, void* out, float* workspace,
                                 const Workspace& wl, hipStream_t stream) {
  const size_t blocks = (size_t)s.B * s.Hkv * (size_t)s.n_chunks;
  if (blocks > 0x7fffffffu || (size_t)s.B * s.Hq > 0x7fffffffu) return hipErrorInvalidConfiguration;
  QParams kp{k.codes, k.scale, k.min, s.k_axis, s.k_group};
  QParams vp{v.codes, v.scale, v.min, s.v_axis, s.v_group};
  float* logits = workspace + wl.logits;
  float* minmax = workspace + wl.minmax;
  float* partial = workspace + wl.partial;
  scores_kernel<<<dim3((unsigned)blocks), dim3(kScoreThreads), 0, stream>>>(
      s, static_cast<const __half*>(q), kp, static_cast<const __half*>(k_text), n_text_dev,
      softmax_scale, logits, minmax);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  pv_kernel<<<dim3((unsigned)blocks), dim3(s.d), 0, stream>>>(
      s, vp, static_cast<const __half*>(v_text), n_text_dev, calib, logits, minmax, partial);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  combine_kernel<<<dim3((unsigned)((size_t)s.B * s.Hq)), dim3(s.d), 0, stream>>>(
      s.n_chunks, s.d, partial, static_cast<__half*>(out));
  return hipGetLastError();
}

}  // namespace cq
