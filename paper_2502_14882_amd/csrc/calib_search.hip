// Grid search of the calibration parameters tau1, tau2 (Sec. 3.2).
//
// For every pair of the grid: the mean squared difference between the attention weights with the
// calibrated logits of the quantized keys, softmax([g(q K_deq^T s), q K_text^T s]), and the
// weights with the exact 16-bit keys, softmax([q K^T s, q K_text^T s]); mean over the attended
// tokens of a query row, then over all (batch, query head) rows.  gamma, delta of g are the
// extrema of the row's visual logits, as in the decode call.  The caller takes the argmin.
//
// A calibration-time utility, not part of the decode step: logits come from the shape-agnostic
// logits kernel (any layout), the weights are formed in fp64.
#include <cfloat>

#include "cq_internal.h"

namespace cq {
namespace {

constexpr int kThreads = 256;

struct TauGrid {
  float tau1[kMaxTauPairs], tau2[kMaxTauPairs];   // pair p = (tau1[p], tau2[p])
  int n_pairs;
};

__device__ inline double block_sum(double v, double* red) {
  __syncthreads();
  red[threadIdx.x] = v;
  __syncthreads();
  for (int off = kThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  return red[0];
}

// grid.x = B * Hq; one block per query row.
__global__ void __launch_bounds__(kThreads)
tau_grid_kernel(int n_vis, int n_text, int chunks_q_vis, int chunks_q, int chunks_x, TauGrid grid,
                const float* __restrict__ logits_q, const float* __restrict__ logits_x,
                const float* __restrict__ minmax_q, const float* __restrict__ minmax_x,
                double* __restrict__ row_mse) {
  __shared__ double red[kThreads];
  const size_t row = blockIdx.x;
  const int n_all = n_vis + n_text;
  const float* sq = logits_q + row * (size_t)n_all;     // visual logits, then text logits
  const float* sx = logits_x + row * (size_t)n_vis;
  // extrema of the row from the chunk extrema of the logits kernel (every thread the same)
  float lo = FLT_MAX, hi = -FLT_MAX, tmax = -FLT_MAX, xmax = -FLT_MAX;
  for (int c = 0; c < chunks_q_vis; ++c) {
    lo = fminf(lo, minmax_q[(row * chunks_q + c) * 2 + 0]);
    hi = fmaxf(hi, minmax_q[(row * chunks_q + c) * 2 + 1]);
  }
  for (int c = chunks_q_vis; c < chunks_q; ++c) tmax = fmaxf(tmax, minmax_q[(row * chunks_q + c) * 2 + 1]);
  for (int c = 0; c < chunks_x; ++c) xmax = fmaxf(xmax, minmax_x[(row * chunks_x + c) * 2 + 1]);
  const double gam = lo, dlt = hi, width = dlt - gam;
  // weights with the exact keys: p_j = exp(s_j - m_ref) / z_ref
  const double m_ref = fmax((double)xmax, (double)tmax);
  double z = 0.0;
  for (int j = threadIdx.x; j < n_all; j += kThreads)
    z += exp((double)(j < n_vis ? sx[j] : sq[j]) - m_ref);
  const double z_ref = block_sum(z, red);

  for (int p = 0; p < grid.n_pairs; ++p) {
    const double t1 = grid.tau1[p], t2 = grid.tau2[p];
    const double slope = width == 0.0 ? 1.0 : (width + t1 - t2) / width;
    const double shift = gam - t1;                 // g(s) = slope * (s - gamma) + gamma - tau1
    // g is monotone: its largest value sits at one end of [gamma, delta]
    const double m_cal = fmax(fmax(shift, slope * width + shift), (double)tmax);
    z = 0.0;
    for (int j = threadIdx.x; j < n_all; j += kThreads) {
      const double s = j < n_vis ? slope * ((double)sq[j] - gam) + shift : (double)sq[j];
      z += exp(s - m_cal);
    }
    const double z_cal = block_sum(z, red);
    double err = 0.0;
    for (int j = threadIdx.x; j < n_all; j += kThreads) {
      const double s = j < n_vis ? slope * ((double)sq[j] - gam) + shift : (double)sq[j];
      const double ref = exp((double)(j < n_vis ? sx[j] : sq[j]) - m_ref) / z_ref;
      const double diff = exp(s - m_cal) / z_cal - ref;
      err += diff * diff;
    }
    const double total = block_sum(err, red);
    if (threadIdx.x == 0) row_mse[row * grid.n_pairs + p] = total / (double)n_all;
  }
}

// One block; thread p sums pair p over the rows in a fixed order.
__global__ void tau_reduce_kernel(int n_rows, int n_pairs, const double* __restrict__ row_mse,
                                  double* __restrict__ mse_out) {
  const int p = threadIdx.x;
  if (p >= n_pairs) return;
  double acc = 0.0;
  for (int r = 0; r < n_rows; ++r) acc += row_mse[(size_t)r * n_pairs + p];
  mse_out[p] = acc / (double)n_rows;
}

}  // namespace

hipError_t launch_tau_search(const DecodeShape& s, const void* q, const void* k_exact,
                             const cq_qtensor_t& k, const void* k_text, const float* tau1,
                             int n_tau1, const float* tau2, int n_tau2, float softmax_scale,
                             double* mse_out, float* workspace, const TauWorkspace& wl,
                             hipStream_t stream) {
  const size_t rows = (size_t)s.B * s.Hq;
  if (rows > 0x7fffffffu || n_tau1 * n_tau2 > kMaxTauPairs) return hipErrorInvalidConfiguration;
  float* logits_q = workspace + wl.logits_q;
  float* logits_x = workspace + wl.logits_x;
  float* minmax_q = workspace + wl.minmax_q;
  float* minmax_x = workspace + wl.minmax_x;
  double* row_mse = reinterpret_cast<double*>(workspace + wl.row_mse);
  // logits on the quantized keys plus the text tail
  hipError_t e = launch_scores_generic(s, q, k, k_text, nullptr, softmax_scale, logits_q, minmax_q, stream);
  if (e != hipSuccess) return e;
  // logits on the exact keys: the same kernel sees them as a 16-bit tail of n_vis tokens
  DecodeShape x = s;
  x.n_vis = 0;
  x.n_text = s.n_vis;
  x.n_text_cap = s.n_vis;
  x.n_vis_chunks = 0;
  x.n_text_chunks = ceil_div(s.n_vis, kTextChunk);
  x.n_chunks = x.n_text_chunks;
  static const cq_qtensor_t kNone = {nullptr, nullptr, nullptr};
  e = launch_scores_generic(x, q, kNone, k_exact, nullptr, softmax_scale, logits_x, minmax_x, stream);
  if (e != hipSuccess) return e;
  TauGrid grid;
  grid.n_pairs = n_tau1 * n_tau2;
  for (int i = 0; i < n_tau1; ++i)
    for (int j = 0; j < n_tau2; ++j) {
      grid.tau1[i * n_tau2 + j] = tau1[i];
      grid.tau2[i * n_tau2 + j] = tau2[j];
    }
  tau_grid_kernel<<<dim3((unsigned)rows), dim3(kThreads), 0, stream>>>(
      s.n_vis, s.n_text, s.n_vis_chunks, s.n_chunks, x.n_chunks, grid, logits_q, logits_x,
      minmax_q, minmax_x, row_mse);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  tau_reduce_kernel<<<dim3(1), dim3(kMaxTauPairs), 0, stream>>>((int)rows, grid.n_pairs, row_mse,
                                                                mse_out);
  return hipGetLastError();
}

}  // namespace cq
