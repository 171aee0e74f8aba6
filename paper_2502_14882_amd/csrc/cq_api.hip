// Host side of libcq: argument validation, kernel-path selection, status strings.
// Every check here runs before the first HIP call, so a rejected call launches nothing.
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "cq_internal.h"

namespace {

thread_local char g_last_error[256] = "";
// test / benchmark switches (cq_bench.h): per thread, never touched by the product calls
thread_local int g_kernel_path = CQ_PATH_AUTO;
thread_local int g_decode_chunks = 0;

int fail(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
  va_end(ap);
  return status;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_group(const char* which, int axis, int group, int n_vis, int d) {
  if (axis == CQ_AXIS_CHANNEL) {
    if (group < 1) return fail(CQ_ERR_SHAPE, "%s_group must be >= 1 (got %d)", which, group);
    if (n_vis % group != 0)
      return fail(CQ_ERR_SHAPE, "n_vis=%d is not a multiple of %s_group=%d", n_vis, which, group);
  } else if (axis == CQ_AXIS_TOKEN) {
    if (group < 32 || group % 32 != 0 || d % group != 0)
      return fail(CQ_ERR_SHAPE,
                  "%s_group=%d must be a multiple of 32 that divides head_dim=%d", which, group, d);
  } else {
    return fail(CQ_ERR_UNSUPPORTED, "%s_axis=%d is not a CQ_AXIS_* value", which, axis);
  }
  return CQ_OK;
}

int check_layout(const cq_layout_t* L, bool need_q_heads, bool need_values = true) {
  if (!L) return fail(CQ_ERR_NULL, "layout is NULL");
  if (L->batch < 1 || L->n_kv_heads < 1)
    return fail(CQ_ERR_SHAPE, "batch=%d and n_kv_heads=%d must be >= 1", L->batch, L->n_kv_heads);
  if (need_q_heads && (L->n_q_heads < 1 || L->n_q_heads % L->n_kv_heads != 0))
    return fail(CQ_ERR_SHAPE, "n_q_heads=%d must be a positive multiple of n_kv_heads=%d",
                L->n_q_heads, L->n_kv_heads);
  if (L->head_dim < 32 || L->head_dim > 256 || L->head_dim % 32 != 0)
    return fail(CQ_ERR_SHAPE, "head_dim=%d must be a multiple of 32 in [32, 256]", L->head_dim);
  if (L->n_vis < 0) return fail(CQ_ERR_SHAPE, "n_vis=%d must be >= 0", L->n_vis);
  if (L->bits != 1 && L->bits != 2 && L->bits != 4 && L->bits != 8)
    return fail(CQ_ERR_UNSUPPORTED, "bits=%d not in {1, 2, 4, 8}", L->bits);
  int rc = check_group("k", L->k_axis, L->k_group, L->n_vis, L->head_dim);
  if (rc != CQ_OK) return rc;
  if (need_values) {
    rc = check_group("v", L->v_axis, L->v_group, L->n_vis, L->head_dim);
    if (rc != CQ_OK) return rc;
  }
  const double elems = (double)L->batch * L->n_kv_heads * (double)L->n_vis * L->head_dim;
  if (elems >= 9.0e18) return fail(CQ_ERR_SHAPE, "tensor too large");
  return CQ_OK;
}

int check_qtensor(const char* which, const cq_qtensor_t* t) {
  if (!t) return fail(CQ_ERR_NULL, "%s is NULL", which);
  if (!t->codes || !t->scale || !t->min)
    return fail(CQ_ERR_NULL, "%s has a NULL codes/scale/min pointer", which);
  if (!aligned16(t->codes) || !aligned16(t->scale) || !aligned16(t->min))
    return fail(CQ_ERR_ALIGN, "%s buffers must be 16-byte aligned", which);
  return CQ_OK;
}

cq::DecodeShape make_shape(const cq_layout_t* L, int n_text, int n_text_cap) {
  cq::DecodeShape s;
  s.B = L->batch; s.Hq = L->n_q_heads; s.Hkv = L->n_kv_heads; s.g = s.Hq / s.Hkv;
  s.d = L->head_dim; s.n_vis = L->n_vis; s.n_text = n_text; s.n_text_cap = n_text_cap;
  s.bits = L->bits; s.k_axis = L->k_axis; s.v_axis = L->v_axis;
  s.k_group = L->k_group; s.v_group = L->v_group;
  s.n_vis_chunks = cq::ceil_div(s.n_vis, cq::kVisChunk);
  s.n_text_chunks = cq::ceil_div(s.n_text, cq::kTextChunk);
  s.n_chunks = s.n_vis_chunks + s.n_text_chunks;
  s.words_per_token = s.d * s.bits / 32;
  return s;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(CQ_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

namespace {
// one new token per (batch, KV head) row into slot n_text of the fp16 tails: 16 bytes per thread
__global__ void __launch_bounds__(256) append_text_kernel(uint4* k_text, uint4* v_text, const uint4* k_new,
                                                          const uint4* v_new, int rows, int n_text,
                                                          int n_text_cap, int vec_per_token) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * vec_per_token) return;
  const int row = i / vec_per_token, c = i % vec_per_token;
  const size_t dst = ((size_t)row * n_text_cap + n_text) * vec_per_token + c;
  k_text[dst] = k_new[i];
  v_text[dst] = v_new[i];
}
// The same with the tail length in device memory: every thread reads it before anyone changes it
// (the increment is a launch of its own, ordered behind this one on the stream).
__global__ void __launch_bounds__(256) append_text_devlen_kernel(uint4* k_text, uint4* v_text, const uint4* k_new,
                                                                 const uint4* v_new, int rows,
                                                                 const int32_t* n_text_dev, int n_text_cap,
                                                                 int vec_per_token) {
  const int n_text = *n_text_dev;
  if (n_text < 0 || n_text >= n_text_cap) return;          // full tail: nothing is written
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * vec_per_token) return;
  const int row = i / vec_per_token, c = i % vec_per_token;
  const size_t dst = ((size_t)row * n_text_cap + n_text) * vec_per_token + c;
  k_text[dst] = k_new[i];
  v_text[dst] = v_new[i];
}
__global__ void bump_tail_length_kernel(int32_t* n_text_dev, int n_text_cap) {
  const int n = *n_text_dev;
  if (n >= 0 && n < n_text_cap) *n_text_dev = n + 1;
}

// Everything cq_decode_attn* checks and decides on the host before the first HIP call.
struct DecodeCall {
  cq::DecodeShape shape;
  cq::Calib calib;
  float softmax_scale;
  bool tuned;               // the tuned kernels run (else the shape-agnostic ones)
  bool streamed;            // tuned, split rows: the streaming kernels with logits kept in scratch
  cq::FusedPlan plan;       // valid when tuned
  cq::StreamPlan stream;    // valid when streamed
  cq::Workspace generic_ws; // valid when !tuned
  size_t ws_bytes;          // scratch the selected kernels touch
};

int check_calib(const cq_calib_t* calib, cq::Calib* c) {
  *c = cq::Calib{CQ_CALIB_NONE, 0.f, 0.f, 0.f, 0.f};
  if (!calib) return CQ_OK;
  if (calib->mode != CQ_CALIB_NONE && calib->mode != CQ_CALIB_DYNAMIC && calib->mode != CQ_CALIB_FIXED)
    return fail(CQ_ERR_UNSUPPORTED, "calib mode %d is not a CQ_CALIB_* value", calib->mode);
  c->mode = calib->mode;
  if (c->mode != CQ_CALIB_NONE) {
    if (!std::isfinite(calib->tau1) || !std::isfinite(calib->tau2))
      return fail(CQ_ERR_SHAPE, "tau1 and tau2 must be finite");
    c->tau1 = calib->tau1;
    c->tau2 = calib->tau2;
  }
  if (c->mode == CQ_CALIB_FIXED) {
    if (!std::isfinite(calib->gamma) || !std::isfinite(calib->delta) || !(calib->delta > calib->gamma))
      return fail(CQ_ERR_SHAPE, "CQ_CALIB_FIXED needs finite delta > gamma");
    c->gamma = calib->gamma;
    c->delta = calib->delta;
  }
  return CQ_OK;
}

// Kernel selection and scratch size for a valid layout: one plan per call, used by the size query,
// by the argument check and by the launch.
// scratch_limit: the most scratch the caller can offer.  Rows that have to be split run on the
// streaming kernels, which keep the raw logits in scratch (2 bytes per query head and visual
// token); when that does not fit the limit they run as chunks of the fused kernel, which form the
// logits twice and keep only extrema and partials.
int select_kernels(const cq_layout_t* L, int n_text, int n_text_cap, size_t scratch_limit,
                   DecodeCall* call) {
  call->shape = make_shape(L, n_text, n_text_cap);
  call->plan = cq::make_fused_plan(call->shape, g_decode_chunks);
  if (g_kernel_path == CQ_PATH_TUNED && !call->plan.ok)
    return fail(CQ_ERR_UNSUPPORTED, "no tuned decode kernel for this layout");
  call->tuned = g_kernel_path != CQ_PATH_GENERIC && call->plan.ok;
  call->streamed = false;
  if (call->tuned && (call->plan.n_chunks > 1 || call->plan.nhb > 1)) {
    call->stream = cq::make_stream_plan(call->shape, g_decode_chunks);
    call->streamed = call->stream.ok && call->stream.ws_bytes <= scratch_limit;
  }
  call->generic_ws = cq::workspace_layout(L->batch, L->n_q_heads, L->head_dim, L->n_vis, n_text);
  call->ws_bytes = call->streamed ? call->stream.ws_bytes
                   : call->tuned  ? call->plan.ws_bytes
                                  : call->generic_ws.total_bytes;
  return CQ_OK;
}

// Argument checks of cq_decode_attn, cq_decode_attn_devlen and the allocation-free variant;
// n_text is the tail length or (n_text_dev != NULL) the host's bound of it.
int check_decode(const cq_layout_t* L, const void* q_f16, const cq_qtensor_t* k,
                 const cq_qtensor_t* v, const void* k_text_f16, const void* v_text_f16,
                 int32_t n_text, int32_t n_text_cap, bool length_on_device,
                 const cq_calib_t* calib, float softmax_scale, const void* out_f16,
                 size_t scratch_limit, DecodeCall* call) {
  int rc = check_layout(L, true);
  if (rc != CQ_OK) return rc;
  if (!q_f16 || !out_f16) return fail(CQ_ERR_NULL, "q_f16 or out_f16 is NULL");
  if (!aligned16(q_f16) || !aligned16(out_f16))
    return fail(CQ_ERR_ALIGN, "q_f16 and out_f16 must be 16-byte aligned");
  if (n_text < 0 || n_text_cap < n_text)
    return fail(CQ_ERR_SHAPE, "need 0 <= n_text (%d) <= n_text_cap (%d)", n_text, n_text_cap);
  if ((long long)L->n_vis + n_text < 1)
    return fail(CQ_ERR_SHAPE, "nothing to attend to: n_vis + n_text == 0");
  if (L->n_vis > 0) {
    if ((rc = check_qtensor("k", k)) != CQ_OK) return rc;
    if ((rc = check_qtensor("v", v)) != CQ_OK) return rc;
  }
  if (n_text > 0 || (length_on_device && n_text_cap > 0)) {
    if (n_text > 0 && (!k_text_f16 || !v_text_f16))
      return fail(CQ_ERR_NULL, "n_text=%d but k_text_f16 or v_text_f16 is NULL", n_text);
    if (!aligned16(k_text_f16) || !aligned16(v_text_f16))
      return fail(CQ_ERR_ALIGN, "text-tail tensors must be 16-byte aligned");
  }
  if ((rc = check_calib(calib, &call->calib)) != CQ_OK) return rc;
  if (!std::isfinite(softmax_scale) || softmax_scale < 0.f)
    return fail(CQ_ERR_SHAPE, "softmax_scale must be finite and >= 0");
  call->softmax_scale = softmax_scale == 0.f ? 1.0f / std::sqrt((float)L->head_dim) : softmax_scale;
  return select_kernels(L, n_text, n_text_cap, scratch_limit, call);
}

int launch_decode(const DecodeCall& call, const void* q_f16, const cq_qtensor_t* k,
                  const cq_qtensor_t* v, const void* k_text_f16, const void* v_text_f16,
                  const int32_t* n_text_dev, void* out_f16, void* workspace, void* stream) {
  static const cq_qtensor_t kNone = {nullptr, nullptr, nullptr};
  const cq_qtensor_t& kq = k ? *k : kNone;
  const cq_qtensor_t& vq = v ? *v : kNone;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const hipError_t e = call.streamed
      ? cq::launch_decode_stream(call.shape, call.stream, q_f16, kq, vq, k_text_f16, v_text_f16,
                                 n_text_dev, call.calib, call.softmax_scale, out_f16,
                                 static_cast<float*>(workspace), st)
      : call.tuned
      ? cq::launch_decode_fused(call.shape, call.plan, q_f16, kq, vq, k_text_f16, v_text_f16,
                                n_text_dev, call.calib, call.softmax_scale, out_f16,
                                static_cast<float*>(workspace), st)
      : cq::launch_decode_generic(call.shape, q_f16, kq, vq, k_text_f16, v_text_f16, n_text_dev,
                                  call.calib, call.softmax_scale, out_f16,
                                  static_cast<float*>(workspace), call.generic_ws, st);
  if (e != hipSuccess) return hip_fail(e, "decode attention");
  return CQ_OK;
}

// Scratch of the allocation-free entry point: part of the library's device image, so every GPU the
// library runs on holds its own copy at its own address until the process ends.  On the host
// this name is only a handle for hipGetSymbolAddress, never an address: kernels and copies get
// the pointer that noalloc_scratch() returns.
static __device__ __align__(256) unsigned char scratch[CQ_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
int noalloc_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(CQ_ERR_HIP, "device index %d is out of range", dev);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u) != 0)
      return fail(CQ_ERR_HIP, "the scratch array has no 256-byte aligned device address");
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // same value from every thread
  }
  *out = p;
  return CQ_OK;
}

int check_workspace(const void* workspace, size_t workspace_bytes, size_t need) {
  if (!workspace) return fail(CQ_ERR_WORKSPACE, "workspace is NULL");
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    return fail(CQ_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < need)
    return fail(CQ_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  return CQ_OK;
}

}  // namespace

extern "C" {

int cq_version(void) { return 200; }

const char* cq_last_error(void) { return g_last_error; }

const char* cq_status_string(int status) {
  switch (status) {
    case CQ_OK: return "CQ_OK";
    case CQ_ERR_NULL: return "CQ_ERR_NULL: a required pointer is NULL";
    case CQ_ERR_SHAPE: return "CQ_ERR_SHAPE: sizes out of range or not divisible";
    case CQ_ERR_UNSUPPORTED: return "CQ_ERR_UNSUPPORTED: bits, axis or group not supported";
    case CQ_ERR_WORKSPACE: return "CQ_ERR_WORKSPACE: workspace missing, misaligned or too small";
    case CQ_ERR_HIP: return "CQ_ERR_HIP: a HIP call or kernel launch failed";
    case CQ_ERR_ALIGN: return "CQ_ERR_ALIGN: a tensor pointer is not 16-byte aligned";
    default: return "unknown cq_status";
  }
}

int cq_bench_set_kernel_path(int path) {
  if (path != CQ_PATH_AUTO && path != CQ_PATH_GENERIC && path != CQ_PATH_TUNED)
    return fail(CQ_ERR_UNSUPPORTED, "unknown kernel path %d", path);
  const int prev = g_kernel_path;
  g_kernel_path = path;
  return prev;
}

int cq_bench_set_decode_chunks(int n_chunks) {
  if (n_chunks < 0) return fail(CQ_ERR_SHAPE, "n_chunks=%d must be >= 0", n_chunks);
  const int prev = g_decode_chunks;
  g_decode_chunks = n_chunks;
  return prev;
}

size_t cq_decode_workspace_bytes(const cq_layout_t* L, int32_t n_text, const cq_calib_t* calib) {
  cq::Calib c;
  if (check_layout(L, true) != CQ_OK || n_text < 0 || check_calib(calib, &c) != CQ_OK) return 0;
  DecodeCall call;
  if (select_kernels(L, n_text, n_text, SIZE_MAX, &call) != CQ_OK) return 0;
  return call.ws_bytes;
}

int cq_quantize_kv(const cq_layout_t* L, const void* k_f16, const void* v_f16,
                   const cq_qtensor_t* k_out, const cq_qtensor_t* v_out, void* stream) {
  int rc = check_layout(L, false);
  if (rc != CQ_OK) return rc;
  const bool do_k = (k_f16 != nullptr) || (k_out != nullptr);
  const bool do_v = (v_f16 != nullptr) || (v_out != nullptr);
  if (!do_k && !do_v) return fail(CQ_ERR_NULL, "both the key and the value pair are NULL");
  if (do_k) {
    if (!k_f16) return fail(CQ_ERR_NULL, "k_f16 is NULL but k_out is not");
    if ((rc = check_qtensor("k_out", k_out)) != CQ_OK) return rc;
    if (!aligned16(k_f16)) return fail(CQ_ERR_ALIGN, "k_f16 must be 16-byte aligned");
  }
  if (do_v) {
    if (!v_f16) return fail(CQ_ERR_NULL, "v_f16 is NULL but v_out is not");
    if ((rc = check_qtensor("v_out", v_out)) != CQ_OK) return rc;
    if (!aligned16(v_f16)) return fail(CQ_ERR_ALIGN, "v_f16 must be 16-byte aligned");
  }
  if (L->n_vis == 0) return CQ_OK;
  const int path = g_kernel_path;
  const bool k_tuned = cq::quantize_tuned_supported(L->n_vis, L->head_dim, L->bits, L->k_axis, L->k_group);
  const bool v_tuned = cq::quantize_tuned_supported(L->n_vis, L->head_dim, L->bits, L->v_axis, L->v_group);
  if (path == CQ_PATH_TUNED && ((do_k && !k_tuned) || (do_v && !v_tuned)))
    return fail(CQ_ERR_UNSUPPORTED, "no tuned quantizer for this layout");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int rows = L->batch * L->n_kv_heads;
  if (do_k) {
    hipError_t e = (path != CQ_PATH_GENERIC && k_tuned)
        ? cq::launch_quantize_tuned(k_f16, *k_out, rows, L->n_vis, L->bits, L->k_axis, L->k_group, s)
        : cq::launch_quantize_generic(k_f16, *k_out, rows, L->n_vis, L->head_dim, L->bits,
                                      L->k_axis, L->k_group, s);
    if (e != hipSuccess) return hip_fail(e, "quantize keys");
  }
  if (do_v) {
    hipError_t e = (path != CQ_PATH_GENERIC && v_tuned)
        ? cq::launch_quantize_tuned(v_f16, *v_out, rows, L->n_vis, L->bits, L->v_axis, L->v_group, s)
        : cq::launch_quantize_generic(v_f16, *v_out, rows, L->n_vis, L->head_dim, L->bits,
                                      L->v_axis, L->v_group, s);
    if (e != hipSuccess) return hip_fail(e, "quantize values");
  }
  return CQ_OK;
}

int cq_decode_attn(const cq_layout_t* L, const void* q_f16, const cq_qtensor_t* k,
                   const cq_qtensor_t* v, const void* k_text_f16, const void* v_text_f16,
                   int32_t n_text, int32_t n_text_cap, const cq_calib_t* calib,
                   float softmax_scale, void* out_f16, void* workspace, size_t workspace_bytes,
                   void* stream) {
  DecodeCall call;
  int rc = check_decode(L, q_f16, k, v, k_text_f16, v_text_f16, n_text, n_text_cap, false, calib,
                        softmax_scale, out_f16, SIZE_MAX, &call);
  if (rc != CQ_OK) return rc;
  if ((rc = check_workspace(workspace, workspace_bytes, call.ws_bytes)) != CQ_OK) return rc;
  return launch_decode(call, q_f16, k, v, k_text_f16, v_text_f16, nullptr, out_f16, workspace, stream);
}

int cq_decode_attn_noalloc(const cq_layout_t* L, const void* q_f16, const cq_qtensor_t* k,
                           const cq_qtensor_t* v, const void* k_text_f16, const void* v_text_f16,
                           int32_t n_text, int32_t n_text_cap, const cq_calib_t* calib,
                           float softmax_scale, void* out_f16, void* stream) {
  DecodeCall call;
  int rc = check_decode(L, q_f16, k, v, k_text_f16, v_text_f16, n_text, n_text_cap, false, calib,
                        softmax_scale, out_f16, (size_t)CQ_NOALLOC_SCRATCH_BYTES, &call);
  if (rc != CQ_OK) return rc;
  if (call.ws_bytes > (size_t)CQ_NOALLOC_SCRATCH_BYTES)
    return fail(CQ_ERR_WORKSPACE,
                "this shape needs %zu bytes of scratch, the allocation-free entry point holds %zu: "
                "call cq_decode_attn with a workspace", call.ws_bytes,
                (size_t)CQ_NOALLOC_SCRATCH_BYTES);
  void* ws = nullptr;
  if ((rc = noalloc_scratch(&ws)) != CQ_OK) return rc;
  return launch_decode(call, q_f16, k, v, k_text_f16, v_text_f16, nullptr, out_f16, ws, stream);
}

int cq_decode_attn_devlen(const cq_layout_t* L, const void* q_f16, const cq_qtensor_t* k,
                          const cq_qtensor_t* v, const void* k_text_f16, const void* v_text_f16,
                          const int32_t* n_text_dev, int32_t n_text_max, int32_t n_text_cap,
                          const cq_calib_t* calib, float softmax_scale, void* out_f16,
                          void* workspace, size_t workspace_bytes, void* stream) {
  if (!n_text_dev) return fail(CQ_ERR_NULL, "n_text_dev is NULL");
  if ((reinterpret_cast<uintptr_t>(n_text_dev) & 3u) != 0)
    return fail(CQ_ERR_ALIGN, "n_text_dev must be 4-byte aligned");
  DecodeCall call;
  int rc = check_decode(L, q_f16, k, v, k_text_f16, v_text_f16, n_text_max, n_text_cap, true, calib,
                        softmax_scale, out_f16, SIZE_MAX, &call);
  if (rc != CQ_OK) return rc;
  if ((rc = check_workspace(workspace, workspace_bytes, call.ws_bytes)) != CQ_OK) return rc;
  return launch_decode(call, q_f16, k, v, k_text_f16, v_text_f16, n_text_dev, out_f16, workspace,
                       stream);
}

size_t cq_tau_search_workspace_bytes(const cq_layout_t* L, int32_t n_text, int32_t n_tau1,
                                     int32_t n_tau2) {
  if (check_layout(L, true, false) != CQ_OK || n_text < 0 || n_tau1 < 1 || n_tau2 < 1 ||
      (long long)n_tau1 * n_tau2 > cq::kMaxTauPairs)
    return 0;
  return cq::tau_workspace_layout(L->batch, L->n_q_heads, L->n_vis, n_text, n_tau1 * n_tau2)
      .total_bytes;
}

int cq_tau_search(const cq_layout_t* L, const void* q_f16, const void* k_exact_f16,
                  const cq_qtensor_t* k, const void* k_text_f16, int32_t n_text, int32_t n_text_cap,
                  const float* tau1, int32_t n_tau1, const float* tau2, int32_t n_tau2,
                  float softmax_scale, double* mse_out, void* workspace, size_t workspace_bytes,
                  void* stream) {
  int rc = check_layout(L, true, false);     // the values play no part
  if (rc != CQ_OK) return rc;
  if (L->n_vis < 1) return fail(CQ_ERR_SHAPE, "no quantized tokens to calibrate: n_vis == 0");
  if (!q_f16 || !k_exact_f16 || !mse_out || !tau1 || !tau2)
    return fail(CQ_ERR_NULL, "q_f16, k_exact_f16, tau1, tau2 or mse_out is NULL");
  if (!aligned16(q_f16) || !aligned16(k_exact_f16))
    return fail(CQ_ERR_ALIGN, "q_f16 and k_exact_f16 must be 16-byte aligned");
  if ((reinterpret_cast<uintptr_t>(mse_out) & 7u) != 0)
    return fail(CQ_ERR_ALIGN, "mse_out must be 8-byte aligned");
  if ((rc = check_qtensor("k", k)) != CQ_OK) return rc;
  if (n_text < 0 || n_text_cap < n_text)
    return fail(CQ_ERR_SHAPE, "need 0 <= n_text (%d) <= n_text_cap (%d)", n_text, n_text_cap);
  if (n_text > 0) {
    if (!k_text_f16) return fail(CQ_ERR_NULL, "n_text=%d but k_text_f16 is NULL", n_text);
    if (!aligned16(k_text_f16)) return fail(CQ_ERR_ALIGN, "k_text_f16 must be 16-byte aligned");
  }
  if (n_tau1 < 1 || n_tau2 < 1 || (long long)n_tau1 * n_tau2 > cq::kMaxTauPairs)
    return fail(CQ_ERR_SHAPE, "the grid needs 1 <= n_tau1 * n_tau2 <= %d pairs (got %d x %d)",
                cq::kMaxTauPairs, n_tau1, n_tau2);
  for (int i = 0; i < n_tau1; ++i)
    if (!std::isfinite(tau1[i])) return fail(CQ_ERR_SHAPE, "tau1[%d] is not finite", i);
  for (int i = 0; i < n_tau2; ++i)
    if (!std::isfinite(tau2[i])) return fail(CQ_ERR_SHAPE, "tau2[%d] is not finite", i);
  if (!std::isfinite(softmax_scale) || softmax_scale < 0.f)
    return fail(CQ_ERR_SHAPE, "softmax_scale must be finite and >= 0");
  if (softmax_scale == 0.f) softmax_scale = 1.0f / std::sqrt((float)L->head_dim);
  const cq::TauWorkspace wl =
      cq::tau_workspace_layout(L->batch, L->n_q_heads, L->n_vis, n_text, n_tau1 * n_tau2);
  if (!workspace) return fail(CQ_ERR_WORKSPACE, "workspace is NULL");
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    return fail(CQ_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < wl.total_bytes)
    return fail(CQ_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes,
                wl.total_bytes);
  const cq::DecodeShape s = make_shape(L, n_text, n_text_cap);
  const hipError_t e = cq::launch_tau_search(s, q_f16, k_exact_f16, *k, k_text_f16, tau1, n_tau1,
                                             tau2, n_tau2, softmax_scale, mse_out,
                                             static_cast<float*>(workspace), wl,
                                             static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "tau search");
  return CQ_OK;
}

static int check_append(const cq_layout_t* L, const void* k_text_f16, const void* v_text_f16,
                        int32_t n_text_cap, const void* k_new_f16, const void* v_new_f16,
                        long long* n_vec, int* vec_per_token) {
  int rc = check_layout(L, false);
  if (rc != CQ_OK) return rc;
  if (!k_text_f16 || !v_text_f16 || !k_new_f16 || !v_new_f16)
    return fail(CQ_ERR_NULL, "a tail or new-token pointer is NULL");
  if (!aligned16(k_text_f16) || !aligned16(v_text_f16) || !aligned16(k_new_f16) ||
      !aligned16(v_new_f16))
    return fail(CQ_ERR_ALIGN, "tails and new-token tensors must be 16-byte aligned");
  if (n_text_cap < 1) return fail(CQ_ERR_SHAPE, "the tail has no capacity: n_text_cap=%d", n_text_cap);
  const long long rows = (long long)L->batch * L->n_kv_heads;
  *vec_per_token = L->head_dim * 2 / 16;          // head_dim is a multiple of 32
  *n_vec = rows * *vec_per_token;
  if (*n_vec > 0x7fffffffLL) return fail(CQ_ERR_SHAPE, "batch * n_kv_heads * head_dim is too large");
  return CQ_OK;
}

int cq_append_text_kv(const cq_layout_t* L, void* k_text_f16, void* v_text_f16, int32_t n_text,
                      int32_t n_text_cap, const void* k_new_f16, const void* v_new_f16,
                      void* stream) {
  long long n;
  int vec_per_token;
  int rc = check_append(L, k_text_f16, v_text_f16, n_text_cap > 0 ? n_text_cap : 1, k_new_f16,
                        v_new_f16, &n, &vec_per_token);
  if (rc != CQ_OK) return rc;
  if (n_text < 0 || n_text >= n_text_cap)
    return fail(CQ_ERR_SHAPE, "the tail is full or n_text is negative: n_text=%d, n_text_cap=%d",
                n_text, n_text_cap);
  append_text_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream)>>>(
      static_cast<uint4*>(k_text_f16), static_cast<uint4*>(v_text_f16),
      static_cast<const uint4*>(k_new_f16), static_cast<const uint4*>(v_new_f16),
      (int)(n / vec_per_token), n_text, n_text_cap, vec_per_token);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(CQ_ERR_HIP, "append_text_kernel: %s", hipGetErrorString(e));
  return CQ_OK;
}

int cq_append_text_kv_devlen(const cq_layout_t* L, void* k_text_f16, void* v_text_f16,
                             int32_t* n_text_dev, int32_t n_text_cap, const void* k_new_f16,
                             const void* v_new_f16, void* stream) {
  long long n;
  int vec_per_token;
  int rc = check_append(L, k_text_f16, v_text_f16, n_text_cap, k_new_f16, v_new_f16, &n,
                        &vec_per_token);
  if (rc != CQ_OK) return rc;
  if (!n_text_dev) return fail(CQ_ERR_NULL, "n_text_dev is NULL");
  if ((reinterpret_cast<uintptr_t>(n_text_dev) & 3u) != 0)
    return fail(CQ_ERR_ALIGN, "n_text_dev must be 4-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  append_text_devlen_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st>>>(
      static_cast<uint4*>(k_text_f16), static_cast<uint4*>(v_text_f16),
      static_cast<const uint4*>(k_new_f16), static_cast<const uint4*>(v_new_f16),
      (int)(n / vec_per_token), n_text_dev, n_text_cap, vec_per_token);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(CQ_ERR_HIP, "append_text_devlen_kernel: %s", hipGetErrorString(e));
  bump_tail_length_kernel<<<dim3(1), dim3(1), 0, st>>>(n_text_dev, n_text_cap);
  e = hipGetLastError();
  if (e != hipSuccess) return fail(CQ_ERR_HIP, "bump_tail_length_kernel: %s", hipGetErrorString(e));
  return CQ_OK;
}

}  // extern "C"
