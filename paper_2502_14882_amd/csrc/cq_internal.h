// Internal declarations shared by the host API and the HIP kernels of libcq.
// Not part of the ABI (see include/cq.h for that).
#ifndef CQ_INTERNAL_H_
#define CQ_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "cq.h"
#include "cq_bench.h"

namespace cq {

// Tokens per block-level work item of the decode pipeline.  A "chunk" is the unit of
// split-K: every chunk produces one (m, l, acc[d]) partial of the online softmax.
constexpr int kVisChunk = 512;
constexpr int kTextChunk = 512;

struct DecodeShape {
  // n_text: tokens of the fp16 tail that are attended, or - when the length lives in device
  // memory (n_text_dev below) - the host's upper bound of it, which sizes launches and buffers
  int B, Hq, Hkv, g, d, n_vis, n_text, n_text_cap;
  int bits, k_axis, v_axis, k_group, v_group;
  int n_vis_chunks, n_text_chunks, n_chunks;
  int words_per_token;  // d * bits / 32
};

// Layout of the caller-provided workspace (all float, offsets in floats).
struct Workspace {
  size_t logits;    // [B][Hq][n_vis + n_text]       raw (uncalibrated) logits
  size_t minmax;    // [B][Hq][n_chunks][2]          min, max of each chunk's logits
  size_t partial;   // [B][Hq][n_chunks][d + 2]      m, l, acc[d]
  size_t total_bytes;
};

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

inline Workspace workspace_layout(int B, int Hq, int d, int n_vis, int n_text) {
  Workspace w;
  const int nvc = ceil_div(n_vis, kVisChunk), ntc = ceil_div(n_text, kTextChunk);
  const size_t rows = (size_t)B * (size_t)Hq;
  auto align64 = [](size_t x) { return (x + 63) / 64 * 64; };
  w.logits = 0;
  w.minmax = align64(w.logits + rows * ((size_t)n_vis + (size_t)n_text));
  w.partial = align64(w.minmax + rows * (size_t)(nvc + ntc) * 2);
  size_t end = align64(w.partial + rows * (size_t)(nvc + ntc) * (size_t)(d + 2));
  w.total_bytes = (end * sizeof(float) + 255) / 256 * 256;
  if (w.total_bytes == 0) w.total_bytes = 256;
  return w;
}

struct Calib {
  int mode;
  float tau1, tau2, gamma, delta;
};

// ---- launchers (each returns the hipError_t of its launches) -----------------------
hipError_t launch_quantize_generic(const void* x_f16, const cq_qtensor_t& out, int rows,
                                   int n_vis, int d, int bits, int axis, int group,
                                   hipStream_t stream);

// n_text_dev (all decode launchers): NULL, or a device int32 holding the current tail length; the
// kernels then attend to min(max(*n_text_dev, 0), s.n_text) text tokens.
hipError_t launch_decode_generic(const DecodeShape& s, const void* q, const cq_qtensor_t& k,
                                 const cq_qtensor_t& v, const void* k_text, const void* v_text,
                                 const int32_t* n_text_dev, const Calib& calib,
                                 float softmax_scale, void* out, float* workspace,
                                 const Workspace& wl, hipStream_t stream);

// First stage of the shape-agnostic decode on its own: raw logits [B*Hq][n_vis + n_text] and the
// extrema [B*Hq][n_chunks][2] of every chunk of tokens.
hipError_t launch_scores_generic(const DecodeShape& s, const void* q, const cq_qtensor_t& k,
                                 const void* k_text, const int32_t* n_text_dev,
                                 float softmax_scale, float* logits, float* minmax,
                                 hipStream_t stream);

// Grid search of the calibration parameters (Sec. 3.2): workspace layout in floats, and launcher.
constexpr int kMaxTauPairs = 64;
struct TauWorkspace {
  size_t logits_q;   // [B*Hq][n_vis + n_text]  logits on the dequantized keys and the text keys
  size_t logits_x;   // [B*Hq][n_vis]           logits on the exact 16-bit keys
  size_t minmax_q;   // [B*Hq][chunks of n_vis + n_text][2]
  size_t minmax_x;   // [B*Hq][chunks of n_vis][2]
  size_t row_mse;    // [B*Hq][n_pairs] doubles
  size_t total_bytes;
};
inline TauWorkspace tau_workspace_layout(int B, int Hq, int n_vis, int n_text, int n_pairs) {
  TauWorkspace w;
  const int nvc = ceil_div(n_vis, kVisChunk), ntc = ceil_div(n_text, kTextChunk);
  // the exact keys go through the text-tail path of the logits kernel: chunks of kTextChunk
  const int nxc = ceil_div(n_vis, kTextChunk);
  const size_t rows = (size_t)B * (size_t)Hq;
  auto align64 = [](size_t x) { return (x + 63) / 64 * 64; };
  w.logits_q = 0;
  w.logits_x = align64(w.logits_q + rows * ((size_t)n_vis + (size_t)n_text));
  w.minmax_q = align64(w.logits_x + rows * (size_t)n_vis);
  w.minmax_x = align64(w.minmax_q + rows * (size_t)(nvc + ntc) * 2);
  w.row_mse = align64(w.minmax_x + rows * (size_t)nxc * 2);
  const size_t end = align64(w.row_mse + rows * (size_t)n_pairs * 2);
  w.total_bytes = (end * sizeof(float) + 255) / 256 * 256;
  return w;
}
hipError_t launch_tau_search(const DecodeShape& s, const void* q, const void* k_exact,
                             const cq_qtensor_t& k, const void* k_text, const float* tau1,
                             int n_tau1, const float* tau2, int n_tau2, float softmax_scale,
                             double* mse_out, float* workspace, const TauWorkspace& wl,
                             hipStream_t stream);

// Register-resident tile quantizer for head_dim 128, b in {1,2,4,8}, n_vis a multiple of 128,
// groups of 32/64/128 or (channel axis) the whole sequence, which adds an extrema pass.
bool quantize_tuned_supported(int n_vis, int d, int bits, int axis, int group);
hipError_t launch_quantize_tuned(const void* x_f16, const cq_qtensor_t& out, int rows, int n_vis,
                                 int bits, int axis, int group, hipStream_t stream);

// Merge the per-chunk partials [n_rows][n_chunks][d + 2] of the online softmax into out.
hipError_t launch_combine(int n_rows, int n_chunks, int d, const float* partial, void* out,
                          hipStream_t stream);

// Tuned decode for head_dim 128 (see decode_fused.hip for the layouts it takes): one fused launch
// when a workgroup can own a whole row, else extrema pass + partial pass + combine over chunks
// of the row.  The plan is made once per call on the host and says what will run.
struct FusedPlan {
  bool ok = false;            // a tuned kernel exists for the shape
  int nhb = 1;                // blocks of 4 query heads per KV head
  int n_chunks = 1;           // chunks per row
  int stride = 0;             // floats between the logit rows of two heads in LDS
  size_t lds = 0;             // dynamic LDS bytes per workgroup
  size_t ws_minmax_floats = 0;  // split rows: [B*Hq][n_chunks][2] (offset of the partials)
  size_t ws_bytes = 256;      // workspace the launches touch (a multiple of 256, >= 256)
};
// min_chunks: 0 = the fewest chunks that fit on chip, n >= 1 = at least n (test override)
FusedPlan make_fused_plan(const DecodeShape& s, int min_chunks);
hipError_t launch_decode_fused(const DecodeShape& s, const FusedPlan& plan, const void* q,
                               const cq_qtensor_t& k, const cq_qtensor_t& v, const void* k_text,
                               const void* v_text, const int32_t* n_text_dev, const Calib& calib,
                               float softmax_scale, void* out, float* workspace,
                               hipStream_t stream);

// Streaming decode for split rows (decode_stream.hip): logits pass (all query heads of a KV head
// per workgroup, raw logits and chunk extrema to the workspace), values pass, combine.  Takes 1- and
// 2-bit codes, keys in groups of 128 tokens, token-wise values, up to 8 query heads per KV head.
struct StreamPlan {
  bool ok = false;
  int ca = 1, cb = 1;              // chunks per row of the logits pass / of the values pass
  int ct = 0;                      // chunks per row of the fp16 tail (values pass)
  size_t ws_lref_floats = 0;       // workspace: [extrema | group references | logits | partials],
  size_t ws_logits_floats = 0;     // offsets in floats
  size_t ws_partial_floats = 0;
  size_t ws_bytes = 256;
};
StreamPlan make_stream_plan(const DecodeShape& s, int min_chunks);
hipError_t launch_decode_stream(const DecodeShape& s, const StreamPlan& plan, const void* q,
                                const cq_qtensor_t& k, const cq_qtensor_t& v, const void* k_text,
                                const void* v_text, const int32_t* n_text_dev, const Calib& calib,
                                float softmax_scale, void* out, float* workspace,
                                hipStream_t stream);

}  // namespace cq

#endif  // CQ_INTERNAL_H_
