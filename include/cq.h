/*
 * cq.h - C ABI of the CalibQuant hot path on MI355X (gfx950).
 *
 * The two operations of the hot path of arxiv 2502.14882:
 *   cq_quantize_kv   uniform b-bit quantization of the visual-token KV cache
 *                    (Sec. 2.2 quantize equation; Sec. 3.1 channel-wise statistics;
 *                    packing appendix), producing packed codes + scale + min;
 *   cq_decode_attn   one decode step of attention that reads the packed cache
 *                    directly (Sec. 3.1 post-scaling, Sec. 3.2 calibration g,
 *                    Sec. 2.1 softmax(.)V), with the 16-bit text-token tail of
 *                    Sec. 3 / Sec. 3.3 ("irregular matrix shape") merged into the
 *                    same softmax;
 * and the steps either side of them:
 *   cq_append_text_kv  growth of the 16-bit tail between decode steps;
 *   cq_tau_search      the grid search of the calibration parameters (Sec. 3.2).
 * (Measurement aids and the test switches live in cq_bench.h, not here.)
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or keeps device memory; it only enqueues kernels.
 *   - All tensors are dense and contiguous in the stated layout, channel (head
 *     dimension) fastest, and 16-byte aligned.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream).  The host structs are read before the call returns.
 *   - Return value: CQ_OK (0) or a negative cq_status.  Argument errors are found on
 *     the host before any HIP call, so nothing is launched when one is returned.
 *     cq_last_error() gives a message for the last failure on the calling thread.
 *   - The library keeps no state between calls beyond that thread-local message (and caches
 *     of device properties); it reads no environment variable.
 *   - Inputs must be finite; NaN/Inf behaviour is undefined (the paper is silent).
 *   - Query head hq attends to KV head hq / (n_q_heads / n_kv_heads).
 */
#ifndef CQ_H_
#define CQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CQ_OK = 0,
  CQ_ERR_NULL = -1,        /* a required pointer is NULL */
  CQ_ERR_SHAPE = -2,       /* sizes do not divide / are out of range */
  CQ_ERR_UNSUPPORTED = -3, /* bits, axis or group not supported */
  CQ_ERR_WORKSPACE = -4,   /* workspace missing, misaligned or too small */
  CQ_ERR_HIP = -5,         /* a HIP call or kernel launch failed */
  CQ_ERR_ALIGN = -6        /* a tensor pointer is not 16-byte aligned */
} cq_status;

/* Which elements share one (min, max) pair - the "statistical range" of Sec. 3.1. */
enum {
  CQ_AXIS_CHANNEL = 0, /* one pair per channel over `group` consecutive tokens
                          (the paper's channel-wise scheme; group = n_vis is the
                          paper's whole-sequence alpha_i, beta_i) */
  CQ_AXIS_TOKEN = 1    /* one pair per token over `group` consecutive channels
                          (the token-wise scheme the paper attributes to KIVI) */
};

/* Problem shape and quantization scheme shared by both calls. */
typedef struct {
  int32_t batch;      /* B  >= 1 */
  int32_t n_q_heads;  /* Hq, a multiple of n_kv_heads (cq_quantize_kv ignores it) */
  int32_t n_kv_heads; /* Hkv >= 1 */
  int32_t head_dim;   /* d: multiple of 32 in [32, 256]; 128 is the tuned case */
  int32_t n_vis;      /* quantized (visual) tokens per sequence, >= 0 */
  int32_t bits;       /* b in {1, 2, 4, 8} */
  int32_t k_axis;     /* CQ_AXIS_* for keys   (hot path: CHANNEL) */
  int32_t v_axis;     /* CQ_AXIS_* for values (hot path: TOKEN) */
  int32_t k_group;    /* CHANNEL axis: tokens per group, divides n_vis;
                         TOKEN axis: channels per group, multiple of 32 dividing d */
  int32_t v_group;    /* same rule, for values */
} cq_layout_t;

/*
 * One quantized tensor of logical shape [B, Hkv, n_vis, d].
 *   codes  uint32 [B, Hkv, n_vis, d*bits/32].  b-bit codes packed along d; element i
 *          of a word sits at bits [32-b(1+i), 32-b*i) (appendix pack(v, N=b, M=32)).
 *   scale  float32, (max-min)/(2^b-1) rounded once to float32.
 *   min    IEEE fp16 bits of the group minimum (a zero is stored as +0).
 *          Shape of scale and min: CHANNEL axis [B, Hkv, n_vis/group, d];
 *                                  TOKEN axis   [B, Hkv, n_vis, d/group].
 * Dequantized element = code * scale + min (Sec. 2.2 dequantize equation).
 */
typedef struct {
  uint32_t *codes;
  float *scale;
  uint16_t *min;
} cq_qtensor_t;

/*
 * Quantize the visual KV cache (Sec. 2.2 + Sec. 3.1 + packing appendix).
 *   k_f16, v_f16  in : fp16 [B, Hkv, n_vis, d]
 *   k_out, v_out  out: buffers of the shapes above, fully overwritten
 * code = round((x - min) * (2^b-1) / (max - min)) evaluated exactly with ties to
 * even; a constant group gives codes 0 and scale 0.  Either of (k_f16, k_out) or
 * (v_f16, v_out) may be NULL as a pair to quantize only the other tensor.
 * n_vis == 0 is a successful no-op.  The output buffers may hold intermediate
 * results until the call's work on `stream` has completed (whole-sequence
 * statistics keep partial extrema in `codes` between their passes); no other
 * memory is touched and nothing is allocated.
 */
int cq_quantize_kv(const cq_layout_t *layout, const void *k_f16, const void *v_f16,
                   const cq_qtensor_t *k_out, const cq_qtensor_t *v_out, void *stream);

/* Calibration of the visual logits (Sec. 3.2):
 *   g(x) = (delta-gamma+tau1-tau2)/(delta-gamma) * (x-gamma) + gamma - tau1. */
enum {
  CQ_CALIB_NONE = 0,    /* g = identity */
  CQ_CALIB_DYNAMIC = 1, /* gamma, delta = min, max of the visual logits of each
                           (batch, query head) row of this call */
  CQ_CALIB_FIXED = 2    /* gamma, delta taken from this struct */
};
typedef struct {
  int32_t mode;
  float tau1, tau2;   /* the paper searches {0,1,2,3}; any finite value is accepted */
  float gamma, delta; /* CQ_CALIB_FIXED only; delta > gamma */
} cq_calib_t;

/* Bytes of scratch cq_decode_attn needs for this shape and calibration (a multiple of 256,
 * > 0): what the kernels that the call will select use.  A row that one workgroup can own
 * (the tuned one-launch kernel) needs the minimum of 256 bytes; a row split over several
 * workgroups needs one (m, l, acc[d]) partial of the online softmax per (batch, query head,
 * chunk), plus the chunks' logit extrema with CQ_CALIB_DYNAMIC; the shape-agnostic kernels
 * also keep one float per (batch, query head, token).  n_text is the largest tail length the
 * workspace has to serve; `calib` may be NULL (= CQ_CALIB_NONE).  Returns 0 if the layout,
 * n_text or the calibration mode is invalid. */
size_t cq_decode_workspace_bytes(const cq_layout_t *layout, int32_t n_text,
                                 const cq_calib_t *calib);

/*
 * One decode step: out = softmax([g(s_vis), s_txt]) [V_deq; V_text]   (Sec. 2.1, 3.2)
 *   s_vis[j] = softmax_scale * q . K_deq[j]  over the n_vis quantized tokens,
 *              computed from the packed codes by post-scaling (Sec. 3.1),
 *   s_txt[t] = softmax_scale * q . K_text[t] over the first n_text text tokens.
 *   q_f16        in : fp16 [B, Hq, d]
 *   k, v         in : quantized visual cache as written by cq_quantize_kv
 *   k_text_f16,
 *   v_text_f16   in : fp16 [B, Hkv, n_text_cap, d]; only the first n_text tokens of
 *                     each head are read; may be NULL when n_text == 0
 *   calib        in : may be NULL (= CQ_CALIB_NONE)
 *   softmax_scale   : 0 means 1/sqrt(d)
 *   out_f16      out: fp16 [B, Hq, d]
 *   workspace       : device scratch of at least cq_decode_workspace_bytes(layout, n_text,
 *                     calib), 256-byte aligned; contents undefined before and after; two
 *                     calls that overlap in time must not share it
 * n_vis + n_text must be >= 1.
 * Errors: CQ_ERR_NULL, CQ_ERR_ALIGN, CQ_ERR_SHAPE, CQ_ERR_UNSUPPORTED (calibration mode),
 * CQ_ERR_WORKSPACE (NULL, misaligned or too small), CQ_ERR_HIP.
 */
int cq_decode_attn(const cq_layout_t *layout, const void *q_f16, const cq_qtensor_t *k,
                   const cq_qtensor_t *v, const void *k_text_f16, const void *v_text_f16,
                   int32_t n_text, int32_t n_text_cap, const cq_calib_t *calib,
                   float softmax_scale, void *out_f16, void *workspace,
                   size_t workspace_bytes, void *stream);

/* Growth of the fp16 tail between decode steps (Sec. 3: only the visual tokens are quantized; the
 * text tokens, including those generated while decoding, stay in 16 bits).  Copies the key and
 * value of ONE new token per sequence, k_new_f16 / v_new_f16 [B, Hkv, 1, d] (device, fp16,
 * 16-byte aligned), to position n_text of the tails k_text_f16 / v_text_f16
 * [B, Hkv, n_text_cap, d] (device, owned by the caller).  The caller then decodes with n_text + 1.
 * Errors: CQ_ERR_NULL, CQ_ERR_ALIGN, CQ_ERR_SHAPE (n_text < 0 or n_text >= n_text_cap),
 * CQ_ERR_HIP.  Asynchronous on `stream`; allocates nothing. */
int cq_append_text_kv(const cq_layout_t *layout, void *k_text_f16, void *v_text_f16,
                      int32_t n_text, int32_t n_text_cap, const void *k_new_f16,
                      const void *v_new_f16, void *stream);

/*
 * cq_decode_attn for callers that cannot allocate or hand over scratch memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * (bit for bit) and errors as cq_decode_attn, without the workspace: whatever scratch the
 * selected kernels need (chunk extrema and online-softmax partials of split rows, logits of the
 * shape-agnostic kernels) lives in an array of CQ_NOALLOC_SCRATCH_BYTES inside the library's
 * device image, one copy per GPU, held until the process ends.  The call allocates and frees
 * nothing; the first call on a device looks the array's address up once (not under capture).
 * A shape that needs more scratch than the array holds (compare
 * cq_decode_workspace_bytes(layout, n_text, calib) with CQ_NOALLOC_SCRATCH_BYTES) returns
 * CQ_ERR_WORKSPACE and launches nothing: use cq_decode_attn with a workspace for it.
 * Every call on a GPU shares that GPU's array and nothing in it needs clearing between calls
 * (each call writes what it reads), but two calls that overlap in time on one GPU - different
 * streams, or different threads - race on it: serialise them, or give them workspaces.
 */
#define CQ_NOALLOC_SCRATCH_BYTES (8u << 20)
int cq_decode_attn_noalloc(const cq_layout_t *layout, const void *q_f16, const cq_qtensor_t *k,
                           const cq_qtensor_t *v, const void *k_text_f16,
                           const void *v_text_f16, int32_t n_text, int32_t n_text_cap,
                           const cq_calib_t *calib, float softmax_scale, void *out_f16,
                           void *stream);

/*
 * The same two steps with the tail length held in DEVICE memory, so that one decode step
 * (append the new token, then attend) can be recorded once into a HIP graph and replayed while
 * the tail grows (Sec. 2.1: every decode step appends the new key and value to the cache).
 *   n_text_dev   : device int32, the current number of text tokens of every sequence.
 *   n_text_max   : HOST upper bound of *n_text_dev for the lifetime of the recording,
 *                  0 <= n_text_max <= n_text_cap.  It sizes the launches, the workspace
 *                  (cq_decode_workspace_bytes(layout, n_text_max, calib)) and the on-chip
 *                  buffers; the kernels read min(max(*n_text_dev, 0), n_text_max) tokens.
 * cq_append_text_kv_devlen writes the new token to slot *n_text_dev of each tail and then
 * increments *n_text_dev; a full tail (*n_text_dev >= n_text_cap) or a negative length leaves
 * the tails and the counter unchanged.  cq_decode_attn_devlen is cq_decode_attn otherwise;
 * n_vis + *n_text_dev must be >= 1 when its kernels run (not checkable on the host).
 * Same errors as the host-length calls, plus CQ_ERR_NULL for n_text_dev and CQ_ERR_ALIGN when
 * it is not 4-byte aligned.  Asynchronous on `stream`; nothing is allocated and nothing is
 * read back to the host.
 */
int cq_append_text_kv_devlen(const cq_layout_t *layout, void *k_text_f16, void *v_text_f16,
                             int32_t *n_text_dev, int32_t n_text_cap, const void *k_new_f16,
                             const void *v_new_f16, void *stream);
int cq_decode_attn_devlen(const cq_layout_t *layout, const void *q_f16, const cq_qtensor_t *k,
                          const cq_qtensor_t *v, const void *k_text_f16, const void *v_text_f16,
                          const int32_t *n_text_dev, int32_t n_text_max, int32_t n_text_cap,
                          const cq_calib_t *calib, float softmax_scale, void *out_f16,
                          void *workspace, size_t workspace_bytes, void *stream);

/* Grid search of the calibration parameters (Sec. 3.2: tau1, tau2 are searched on a grid once and
 * then fixed).  For every pair (tau1[i], tau2[j]) computes the mean squared difference between
 * the attention weights softmax([g(q K_deq^T s), q K_text^T s]) over the quantized keys `k`, with
 * gamma, delta the extrema of each row's visual logits as in CQ_CALIB_DYNAMIC, and the weights
 * softmax([q K^T s, q K_text^T s]) over the exact keys; the mean runs over the n_vis + n_text
 * attended tokens of a query row and then over the B * Hq rows (the error measure of the section's
 * second figure).  The caller takes the argmin.
 *   q_f16        in : fp16 [B, Hq, d] (device)
 *   k_exact_f16  in : fp16 [B, Hkv, n_vis, d] (device), the keys that `k` quantizes
 *   k            in : quantized keys of `layout` (device)
 *   k_text_f16   in : fp16 [B, Hkv, n_text_cap, d] (device); may be NULL when n_text == 0
 *   tau1, tau2   in : HOST arrays of n_tau1 and n_tau2 finite values, read before the call
 *                     returns; 1 <= n_tau1 * n_tau2 <= 64
 *   softmax_scale   : 0 means 1/sqrt(d)
 *   mse_out      out: double [n_tau1][n_tau2] (device, 8-byte aligned)
 *   workspace       : device scratch of at least cq_tau_search_workspace_bytes(), 256-byte
 *                     aligned (the logits of both key sets: 4 * B * Hq * (2 n_vis + n_text) bytes
 *                     and a little more)
 * Works for every layout of the keys; the values play no part.  A calibration-time utility: its
 * kernels are plain (fp64 weights).  Errors: CQ_ERR_NULL, CQ_ERR_ALIGN, CQ_ERR_SHAPE (n_vis == 0,
 * grid size, non-finite tau), CQ_ERR_WORKSPACE, CQ_ERR_HIP.  Asynchronous on `stream`; allocates
 * nothing.  cq_tau_search_workspace_bytes returns 0 for an invalid layout or grid. */
size_t cq_tau_search_workspace_bytes(const cq_layout_t *layout, int32_t n_text, int32_t n_tau1,
                                     int32_t n_tau2);
int cq_tau_search(const cq_layout_t *layout, const void *q_f16, const void *k_exact_f16,
                  const cq_qtensor_t *k, const void *k_text_f16, int32_t n_text,
                  int32_t n_text_cap, const float *tau1, int32_t n_tau1, const float *tau2,
                  int32_t n_tau2, float softmax_scale, double *mse_out, void *workspace,
                  size_t workspace_bytes, void *stream);

/* Text for a cq_status value; never NULL. */
const char *cq_status_string(int status);
/* Message of the last failure on this thread ("" if none). */
const char *cq_last_error(void);
/* ABI version: major*10000 + minor*100 + patch. */
int cq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CQ_H_ */
