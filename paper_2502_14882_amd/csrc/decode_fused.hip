// Fused decode attention over the packed 1-bit cache for head_dim 128 (gfx950).
//
// One workgroup owns one (batch, KV head) row: all of its g query heads, every visual token and
// the text tail.  The raw logits of the row live in LDS, so the dynamic calibration of Sec. 3.2
// (whose gamma, delta are the extrema of ALL visual logits of a query row) needs no second pass
// over memory: phase 1 computes logits and their extrema, phase 2 exponentiates g(s) and
// accumulates the weighted value sum.
//
// Both contractions run on the int8 matrix cores (v_mfma_i32_16x16x64_i8) without ever
// dequantizing an element:
//   * a packed word AND (0x01010101 << p) is already a valid int8 operand: four channels whose
//     byte is 0 or 2^p (-128 for p = 7).  Eight ANDs expand a 32-channel word;
//   * the other operand carries the post-scaled query of Sec. 3.1, q * scale_t * softmax_scale
//     (resp. the weights p_j * scale_j for the values), as a 32-bit fixed-point number split into
//     four signed base-256 digits that sit in four matrix rows; the power of two of the bit
//     position is folded into that operand (keys) or divided out of the result column (values);
//   * operands that have to be transposed between "one lane per row" and "one lane per column"
//     go through LDS and come back with ds_read_b64_tr_b8, which hands lane l the l-th byte of
//     eight 16-byte rows.  A token's 128 one-bit codes are exactly one such row.
// The additive term of post-scaling (q . min_t, resp. sum_j p_j min_j) stays in fp32.
#include <hip/hip_fp16.h>

#include <cfloat>

#include "cq_internal.h"

namespace cq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int kD = 128;            // head_dim
constexpr int kThreads = 512;      // 8 waves; equals kHeads * kD (one query element each)
constexpr int kWaves = kThreads / 64;
constexpr int kHeads = 4;          // query heads per matrix pass (4 digits x 4 heads = 16 rows)
constexpr int kStageBytes = 2048;  // per-wave LDS staging
constexpr float kLog2e = 1.4426950408889634f;

struct FusedArgs {
  const __half* q;
  const uint32_t* k_codes; const float* k_scale; const uint16_t* k_min;
  const uint32_t* v_codes; const float* v_scale; const uint16_t* v_min;
  const __half* k_text; const __half* v_text;
  __half* out;
  int Hq, Hkv, g, n_vis, n_text, n_text_cap, k_group;
  int stride;        // floats between the logit rows of two heads in LDS
  int calib_mode; float tau1, tau2, gamma, delta, softmax_scale;
#ifdef CQ_PHASE_CLOCKS
  long long* clocks;   // [rows][16] time stamps of the phase boundaries (profiling builds only)
#endif
};

#ifdef CQ_PHASE_CLOCKS
#define CQ_CLK(k) do { if (tid == 0 && a.clocks) a.clocks[(size_t)row * 16 + (k)] = wall_clock64(); } while (0)
#else
#define CQ_CLK(k) do { } while (0)
#endif

__device__ inline v2i lds_read_tr8(const uint8_t* p) {
  return __builtin_amdgcn_ds_read_tr8_b64_v2i32(
      (__attribute__((address_space(3))) v2i*)(p));
}

// x -> four signed base-256 digits stored as the four bytes of the result.
__device__ inline int signed_digits(int x) { return (x + 0x00808080) ^ 0x00808080; }

__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_min(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Largest F with bound * 2^F <= 2^29, clamped so that 2^(F-7) and 2^-F stay normal floats.
__device__ inline int fixed_point_shift(float bound) {
  if (!(bound > 0.f)) return 0;
  int e;
  frexpf(bound, &e);           // bound = m * 2^e, m in [0.5, 1)
  return max(-90, min(90, 29 - e));
}

extern __shared__ __align__(16) uint8_t smem[];

// TILES = 16-token tiles per key group (k_group / 16).
template <int TILES>
__global__ void __launch_bounds__(kThreads)
fused_row_kernel(const FusedArgs a) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;                 // b * Hkv + kvh
  const int b = row / a.Hkv, kvh = row % a.Hkv;
  const int n_groups = a.n_vis / a.k_group;
  const int n_all = a.n_vis + a.n_text;

  CQ_CLK(0);
  // ---- LDS carve-up
  float* logits = reinterpret_cast<float*>(smem);                       // [kHeads][stride]
  size_t off = (size_t)kHeads * a.stride * sizeof(float);
  if (off < (size_t)kWaves * kHeads * kD * sizeof(float)) off = (size_t)kWaves * kHeads * kD * sizeof(float);
  float* qf = reinterpret_cast<float*>(smem + off);   off += kHeads * kD * sizeof(float);
  float* bias = reinterpret_cast<float*>(smem + off); off += (size_t)kHeads * max(n_groups, 1) * sizeof(float);
  off = (off + 15) & ~(size_t)15;
  uint8_t* stage = smem + off + (size_t)wave * kStageBytes; off += (size_t)kWaves * kStageBytes;
  float* red = reinterpret_cast<float*>(smem + off);   // [kWaves][kHeads][6]

  // rows of unused heads (g < 4) are computed along but never output; keep them finite
  for (int i = a.g * a.stride + tid; i < kHeads * a.stride; i += kThreads) logits[i] = 0.f;
  // ---- phase 0: query to LDS, fixed-point ranges, additive post-scaling term.
  // The first batch of every metadata stream is requested before anything waits.
  const float* ks_row = a.k_scale + (size_t)row * n_groups * kD;
  const uint16_t* km_row = a.k_min + (size_t)row * n_groups * kD;
  const float* vs_row = a.v_scale + (size_t)row * a.n_vis;
  const uint16_t* vm_row = a.v_min + (size_t)row * a.n_vis;
  const int N4 = n_groups * (kD / 4), N8 = n_groups * (kD / 8), NV4 = a.n_vis / 4;
  constexpr int U4 = 4, U8 = 2;
  v4f ksb[U4], vsb[U4];
  v8h kmb[U8];
  if (a.n_vis > 0) {
#pragma unroll
    for (int u = 0; u < U4; ++u) {
      ksb[u] = *reinterpret_cast<const v4f*>(ks_row + (size_t)min(tid + u * kThreads, N4 - 1) * 4);
      vsb[u] = *reinterpret_cast<const v4f*>(vs_row + (size_t)min(tid + u * kThreads, NV4 - 1) * 4);
    }
#pragma unroll
    for (int u = 0; u < U8; ++u)
      kmb[u] = *reinterpret_cast<const v8h*>(km_row + (size_t)min(tid + u * kThreads, N8 - 1) * 8);
  }
  {
    const int h = tid / kD, c = tid % kD;        // kThreads == kHeads * kD
    qf[tid] = h < a.g ? __half2float(a.q[((size_t)b * a.Hq + (size_t)kvh * a.g + h) * kD + c]) : 0.f;
  }
  __syncthreads();
  float amax[kHeads] = {0.f, 0.f, 0.f, 0.f};
  for (int base = 0; base < N4; base += U4 * kThreads) {
#pragma unroll
    for (int u = 0; u < U4; ++u) {
      const int e4 = base + tid + u * kThreads;
      if (base > 0)
        ksb[u] = *reinterpret_cast<const v4f*>(ks_row + (size_t)min(e4, N4 - 1) * 4);
      if (e4 < N4) {
        const int c = (e4 % (kD / 4)) * 4;
#pragma unroll
        for (int h = 0; h < kHeads; ++h) {
          const v4f qq = *reinterpret_cast<const v4f*>(qf + h * kD + c);
#pragma unroll
          for (int i = 0; i < 4; ++i) amax[h] = fmaxf(amax[h], fabsf(qq[i] * ksb[u][i]));
        }
      }
    }
  }
  for (int base = 0; base < N8; base += U8 * kThreads) {
#pragma unroll
    for (int u = 0; u < U8; ++u) {
      const int e8 = base + tid + u * kThreads;
      if (base > 0)
        kmb[u] = *reinterpret_cast<const v8h*>(km_row + (size_t)min(e8, N8 - 1) * 8);
      if (e8 < N8) {          // the 16 lanes that share a token group enter together
        const int t = e8 / (kD / 8), c0 = (e8 % (kD / 8)) * 8;
        float part[kHeads];
#pragma unroll
        for (int h = 0; h < kHeads; ++h) {
          float sacc = 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) sacc = fmaf(qf[h * kD + c0 + i], (float)kmb[u][i], sacc);
          part[h] = sacc;
        }
#pragma unroll
        for (int h = 0; h < kHeads; ++h) {
          float sacc = part[h];
          for (int o = 8; o > 0; o >>= 1) sacc += __shfl_xor(sacc, o);
          if ((lane & 15) == 0) bias[h * n_groups + t] = sacc * a.softmax_scale;
        }
      }
    }
  }
  float vmax = 0.f;
  for (int base = 0; base < NV4; base += U4 * kThreads) {
#pragma unroll
    for (int u = 0; u < U4; ++u) {
      const int j4 = base + tid + u * kThreads;
      if (base > 0)
        vsb[u] = *reinterpret_cast<const v4f*>(vs_row + (size_t)min(j4, NV4 - 1) * 4);
      if (j4 < NV4)
        vmax = fmaxf(fmaxf(vmax, fmaxf(vsb[u][0], vsb[u][1])), fmaxf(vsb[u][2], vsb[u][3]));
    }
  }
#pragma unroll
  for (int h = 0; h < kHeads; ++h) amax[h] = wave_max(amax[h]);
  vmax = wave_max(vmax);
  if (lane == 0) {
    for (int h = 0; h < kHeads; ++h) red[(wave * kHeads + h) * 6 + 0] = amax[h];
    red[(wave * kHeads) * 6 + 1] = vmax;
  }
  __syncthreads();
  int Fk[kHeads];
#pragma unroll
  for (int h = 0; h < kHeads; ++h) {
    float m = 0.f;
    for (int w = 0; w < kWaves; ++w) m = fmaxf(m, red[(w * kHeads + h) * 6 + 0]);
    Fk[h] = fixed_point_shift(m * a.softmax_scale);
  }
  int Fv;
  {
    float m = 0.f;
    for (int w = 0; w < kWaves; ++w) m = fmaxf(m, red[(w * kHeads) * 6 + 1]);
    Fv = fixed_point_shift(m);
  }
  __syncthreads();   // red is reused below
  CQ_CLK(1);

  // ---- phase 1a: visual logits.  Lane roles:
  //   writer of the query operand: lane handles two 16-byte LDS rows (two channels, all heads)
  //   matrix lane (n = lane % 16, kb = lane / 16): token n of a 16-token tile, word kb of it;
  //   result lane: token n, head lane / 16 (its four digits are the lane's four accumulators)
  const int n16 = lane & 15, kb = lane >> 4;
  const int hres = kb;                       // head whose logits this lane finishes
  float mn = FLT_MAX, mx = -FLT_MAX;
  if (a.n_vis > 0) {
    // writer constants: LDS row r = ((kb*2 + i)*4 + v)*4 + y  <->  channel 32kb + 31 - (4i+v) - 8y
    const int wkb = lane >> 4, wi = (lane >> 3) & 1, wv = (lane >> 1) & 3, wy = (lane & 1) * 2;
    const int wp = 4 * wi + wv;
    const int wc0 = 32 * wkb + 31 - wp - 8 * wy, wc1 = wc0 - 8;
    float qv0[kHeads], qv1[kHeads];
#pragma unroll
    for (int h = 0; h < kHeads; ++h) {
      const float f = ldexpf(a.softmax_scale, Fk[h] - wp) * (wp == 7 ? -1.f : 1.f);
      qv0[h] = qf[h * kD + wc0] * f;
      qv1[h] = qf[h * kD + wc1] * f;
    }
    const float inv_f = ldexpf(1.f, -Fk[hres]);
    const uint32_t* kc_lane = a.k_codes + (size_t)row * a.n_vis * 4 + n16 * 4 + kb;
    const uint8_t* a_addr = stage + (size_t)(kb * 32 + (n16 >> 1)) * 16 + (n16 & 1) * 8;
    float* lrow = logits + (size_t)hres * a.stride + n16;
    // software pipeline: the words and scales of the wave's next group are in flight while the
    // current group is on the matrix cores
    uint32_t wc[TILES], wn[TILES];
    float s0 = 0.f, s1 = 0.f, s0n = 0.f, s1n = 0.f;
    int t = wave;
    if (t < n_groups) {
#pragma unroll
      for (int i = 0; i < TILES; ++i) wc[i] = kc_lane[((size_t)t * TILES + i) * 64];
      s0 = ks_row[(size_t)t * kD + wc0];
      s1 = ks_row[(size_t)t * kD + wc1];
    }
    for (; t < n_groups; t += kWaves) {
      // clamped instead of guarded: a branch here would make the compiler wait for these
      // loads at the join, i.e. before the current group is even started
      const int tn = min(t + kWaves, n_groups - 1);
#pragma unroll
      for (int i = 0; i < TILES; ++i) wn[i] = kc_lane[((size_t)tn * TILES + i) * 64];
      s0n = ks_row[(size_t)tn * kD + wc0];
      s1n = ks_row[(size_t)tn * kD + wc1];
      v4i x0, x1;
#pragma unroll
      for (int h = 0; h < kHeads; ++h) {
        x0[h] = signed_digits(__float2int_rn(qv0[h] * s0));
        x1[h] = signed_digits(__float2int_rn(qv1[h] * s1));
      }
      __builtin_amdgcn_wave_barrier();
      *reinterpret_cast<v4i*>(stage + (size_t)lane * 32) = x0;
      *reinterpret_cast<v4i*>(stage + (size_t)lane * 32 + 16) = x1;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      // A operand of matrix i: rows (kb*2 + i)*16 .. +15, two transposing reads of 8 rows
      v2i r00 = lds_read_tr8(a_addr), r01 = lds_read_tr8(a_addr + 128);
      v2i r10 = lds_read_tr8(a_addr + 256), r11 = lds_read_tr8(a_addr + 384);
      const v4i A0 = {r00[0], r00[1], r01[0], r01[1]};
      const v4i A1 = {r10[0], r10[1], r11[0], r11[1]};
      const float bias_h = bias[hres * n_groups + t];
#pragma unroll
      for (int tile = 0; tile < TILES; ++tile) {
        const uint32_t w = wc[tile];
        v4i B0, B1;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          B0[v] = (int)(w & (0x01010101u << v));
          B1[v] = (int)(w & (0x01010101u << (4 + v)));
        }
        v4i c = {0, 0, 0, 0};
        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(A0, B0, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(A1, B1, c, 0, 0, 0);
        const int lo = c[0] + (c[1] << 8), hi = c[2] + (c[3] << 8);
        const float sv = fmaf(fmaf((float)hi, 65536.f, (float)lo), inv_f, bias_h);
        // lanes of unused heads (hres >= g) see q = 0, finish with sv = 0 and write their own
        // (never read) logit row: no branch in the hot loop
        lrow[(t * TILES + tile) * 16] = sv;
        mn = fminf(mn, sv);
        mx = fmaxf(mx, sv);
      }
#pragma unroll
      for (int i = 0; i < TILES; ++i) wc[i] = wn[i];
      s0 = s0n;
      s1 = s1n;
    }
  }

  CQ_CLK(2);
  // ---- phase 1b: text logits on the fp16 matrix cores (products of fp16 numbers are exact)
  if (a.n_text > 0) {
    v8h At[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        At[s][i] = n16 < a.g ? (_Float16)qf[n16 * kD + 32 * kb + 8 * s + i] : (_Float16)0;
    const __half* kt_row = a.k_text + (size_t)row * a.n_text_cap * kD;
    for (int t0 = wave * 16; t0 < a.n_text; t0 += 2 * kWaves * 16) {
      v8h kt[2][4];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int tok = min(t0 + u * kWaves * 16 + n16, a.n_text - 1);
        const v8h* src = reinterpret_cast<const v8h*>(kt_row + (size_t)tok * kD + 32 * kb);
#pragma unroll
        for (int s = 0; s < 4; ++s) kt[u][s] = src[s];
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        v4f c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 4; ++s)
          c = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[s], kt[u][s], c, 0, 0, 0);
        const int tok = t0 + u * kWaves * 16 + n16;
        // rows 4*kb + r = head; only lane groups with heads < g matter
        if (tok < a.n_text) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int h = 4 * kb + r;
            if (h < a.g) logits[h * a.stride + a.n_vis + tok] = c[r] * a.softmax_scale;
          }
        }
      }
    }
  }
  CQ_CLK(3);
  // visual extrema: each lane holds those of head hres over its tokens; fold the 16 token lanes
  mn = fminf(mn, __shfl_xor(mn, 8)); mx = fmaxf(mx, __shfl_xor(mx, 8));
  mn = fminf(mn, __shfl_xor(mn, 4)); mx = fmaxf(mx, __shfl_xor(mx, 4));
  mn = fminf(mn, __shfl_xor(mn, 2)); mx = fmaxf(mx, __shfl_xor(mx, 2));
  mn = fminf(mn, __shfl_xor(mn, 1)); mx = fmaxf(mx, __shfl_xor(mx, 1));
  if (n16 == 0) {
    red[(wave * kHeads + hres) * 6 + 0] = mn;
    red[(wave * kHeads + hres) * 6 + 1] = mx;
  }
  __syncthreads();
  // text maxima: thread-strided scan of the text logits in LDS (n_text is small)
  {
    float tm[kHeads];
#pragma unroll
    for (int h = 0; h < kHeads; ++h) {
      tm[h] = -FLT_MAX;
      if (h < a.g)
        for (int j = tid; j < a.n_text; j += kThreads)
          tm[h] = fmaxf(tm[h], logits[h * a.stride + a.n_vis + j]);
      tm[h] = wave_max(tm[h]);
    }
    if (lane == 0)
      for (int h = 0; h < kHeads; ++h) red[(wave * kHeads + h) * 6 + 2] = tm[h];
  }
  __syncthreads();

  CQ_CLK(4);
  // ---- phase 2 set-up: calibration line and the softmax reference point, per head
  float a2[kHeads], c2v[kHeads], c2t[kHeads];
#pragma unroll
  for (int h = 0; h < kHeads; ++h) {
    float lo = FLT_MAX, hi = -FLT_MAX, tm = -FLT_MAX;
    for (int w = 0; w < kWaves; ++w) {
      lo = fminf(lo, red[(w * kHeads + h) * 6 + 0]);
      hi = fmaxf(hi, red[(w * kHeads + h) * 6 + 1]);
      tm = fmaxf(tm, red[(w * kHeads + h) * 6 + 2]);
    }
    float slope = 1.f, gam = 0.f, shift = 0.f;    // s' = slope * (s - gam) + shift
    if (a.calib_mode != CQ_CALIB_NONE && a.n_vis > 0) {
      float glo = a.gamma, ghi = a.delta;
      if (a.calib_mode == CQ_CALIB_DYNAMIC) { glo = lo; ghi = hi; }
      const float width = ghi - glo;
      slope = width == 0.f ? 1.f : (width + a.tau1 - a.tau2) / width;
      gam = glo;
      shift = glo - a.tau1;
    }
    float M = tm;
    if (a.n_vis > 0) {
      M = fmaxf(M, slope * (lo - gam) + shift);
      M = fmaxf(M, slope * (hi - gam) + shift);
    }
    a2[h] = slope * kLog2e;
    c2v[h] = (shift - slope * gam - M) * kLog2e;
    c2t[h] = -M * kLog2e;
  }

  CQ_CLK(5);
  // ---- phase 2a: weighted value sum over the visual tokens, 64 tokens per step
  v4i acc[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) acc[p] = (v4i){0, 0, 0, 0};
  float lsum[kHeads] = {0.f, 0.f, 0.f, 0.f}, msum[kHeads] = {0.f, 0.f, 0.f, 0.f};
  if (a.n_vis > 0) {
    // Pipeline over 64-token tiles (tile i of this wave = tokens j0 + i * 512 ...):
    //   G(i)  global loads of the tile's codes, scale and min into registers
    //   P(i)  weights p = 2^(a2*s + c2) from the logits in LDS, their fixed-point digits X(i)
    //         and the raw code bytes back to LDS
    //   M(i)  transposing reads of X(i) and the codes, 8 x (4 AND + 1 MFMA)
    // One loop trip runs M(i), P(i+1) and G(i+2); M(i) and P(i+1) are independent, so the
    // matrix pipe and the VALU overlap.  X(i) overwrites the tile's own logits (1 KB for
    // 4 heads x 64 tokens, dead once read), the code bytes alternate between two 1 KB buffers.
    const float fv = ldexpf(1.f, Fv);
    const uint32_t* vc_row = a.v_codes + (size_t)row * a.n_vis * 4;
    const int step = kWaves * 64;
    const int last = a.n_vis - 64;                // first token of the row's last tile
    // per-lane byte offsets inside a tile's staging areas
    const int x_wr = ((lane >> 4) * a.stride) * 4 + (lane & 15) * 16;          // row of token lane
    const int x_rd = (kb * a.stride) * 4 + (n16 >> 1) * 16 + (n16 & 1) * 8;   // tr rows 16kb+k
    const int v_rd = (kb * 16 + (n16 >> 1)) * 16 + (n16 & 1) * 8;
    uint8_t* lbytes = reinterpret_cast<uint8_t*>(logits);

    int j0 = wave * 64;
    v4i cg1, cg2;            // G registers: tile i+1 (ready for P), tile i+2 (in flight)
    float vs1, vm1, vs2, vm2;
    auto load_tile = [&](int jt, v4i& c, float& sc, float& mnv) {
      const int j = min(jt, last) + lane;         // clamped: never a branch around a load
      c = *reinterpret_cast<const v4i*>(vc_row + (size_t)j * 4);
      sc = vs_row[j];
      mnv = __half2float(__ushort_as_half(vm_row[j]));
    };
    auto prep_tile = [&](int jt, int buf, const v4i& c, float sc, float mnv) {
      const float vsf = sc * fv;
      float lg[kHeads];
#pragma unroll
      for (int h = 0; h < kHeads; ++h) lg[h] = logits[h * a.stride + jt + lane];
      v4i xs;
#pragma unroll
      for (int h = 0; h < kHeads; ++h) {
        const float p = __builtin_amdgcn_exp2f(fmaf(lg[h], a2[h], c2v[h]));
        lsum[h] += p;
        msum[h] = fmaf(p, mnv, msum[h]);
        xs[h] = signed_digits(__float2int_rn(p * vsf));
      }
      *reinterpret_cast<v4i*>(lbytes + (size_t)jt * 4 + x_wr) = xs;
      *reinterpret_cast<v4i*>(stage + buf * 1024 + lane * 16) = c;
    };
    if (j0 < a.n_vis) {
      load_tile(j0, cg1, vs1, vm1);
      load_tile(j0 + step, cg2, vs2, vm2);
      prep_tile(j0, 0, cg1, vs1, vm1);
      cg1 = cg2; vs1 = vs2; vm1 = vm2;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    int buf = 0;
    for (; j0 < a.n_vis; j0 += step, buf ^= 1) {
      // M(i): operands of the current tile
      const uint8_t* xr = lbytes + (size_t)j0 * 4 + x_rd;
      const uint8_t* vr = stage + buf * 1024 + v_rd;
      const v2i a_lo = lds_read_tr8(xr), a_hi = lds_read_tr8(xr + 128);
      const v2i b_lo = lds_read_tr8(vr), b_hi = lds_read_tr8(vr + 128);
      const v4i A = {a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
      const v4i raw = {b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
      // G(i+2)
      load_tile(j0 + 2 * step, cg2, vs2, vm2);
      // P(i+1)  (wave-uniform guard: only the LDS traffic is skipped past the end)
      if (j0 + step < a.n_vis) prep_tile(j0 + step, buf ^ 1, cg1, vs1, vm1);
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        v4i B;
#pragma unroll
        for (int v = 0; v < 4; ++v) B[v] = raw[v] & (int)(0x01010101u << p);
        acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, B, acc[p], 0, 0, 0);
      }
      cg1 = cg2; vs1 = vs2; vm1 = vm2;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
  CQ_CLK(6);
  __syncthreads();    // every wave is done reading the logits of the visual tokens
  CQ_CLK(7);

  // ---- phase 2b: per-wave partial output [head][channel] in LDS (reusing the logit area is
  // not possible yet: the text logits are still needed), so partials go to a separate pass:
  // first the text tail is accumulated in registers, then all partials are written.
  // Text tail: lane owns channels 2*lane, 2*lane+1 for all heads.
  // lane = (token slot lane / 16, channels 8 * (lane % 16) .. +7): one 16-byte load covers
  // 8 channels of one token, a wave-wide load covers 4 tokens
  float tacc[kHeads][8];
  float tl[kHeads] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int h = 0; h < kHeads; ++h)
#pragma unroll
    for (int i = 0; i < 8; ++i) tacc[h][i] = 0.f;
  if (a.n_text > 0) {
    const __half* vt_row = a.v_text + (size_t)row * a.n_text_cap * kD + 8 * n16;
    v4f* pw = reinterpret_cast<v4f*>(stage);       // [64 tokens] weights of the 4 heads
    for (int t0 = wave * 64; t0 < a.n_text; t0 += kWaves * 64) {
      const int nt = min(64, a.n_text - t0);
      v4f pv = {0.f, 0.f, 0.f, 0.f};
      if (lane < nt) {
#pragma unroll
        for (int h = 0; h < kHeads; ++h)
          if (h < a.g)
            pv[h] = __builtin_amdgcn_exp2f(
                fmaf(logits[h * a.stride + a.n_vis + t0 + lane], kLog2e, c2t[h]));
      }
#pragma unroll
      for (int h = 0; h < kHeads; ++h) tl[h] += pv[h];
      __builtin_amdgcn_wave_barrier();
      pw[lane] = pv;                               // zero beyond nt
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      for (int u = 0; u < nt; u += 16) {           // 4 wave-wide loads = 16 tokens per trip
        v8h raw[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
          raw[i] = *reinterpret_cast<const v8h*>(
              vt_row + (size_t)(t0 + min(u + 4 * i + kb, nt - 1)) * kD);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const v4f pp = pw[min(u + 4 * i + kb, 63)];      // zero weight for clamped tokens
#pragma unroll
          for (int h = 0; h < kHeads; ++h)
#pragma unroll
            for (int c = 0; c < 8; ++c) tacc[h][c] = fmaf(pp[h], (float)raw[i][c], tacc[h][c]);
        }
      }
    }
    // fold the four token slots
#pragma unroll
    for (int h = 0; h < kHeads; ++h)
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        float v = tacc[h][c];
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 32);
        tacc[h][c] = v;
      }
  }
  CQ_CLK(8);
  __syncthreads();    // logits are dead from here on; their LDS becomes the partial buffer
  CQ_CLK(9);

  float* partial = reinterpret_cast<float*>(smem) + (size_t)wave * kHeads * kD;   // [head][channel]
  {
    // matrix result lane: column n16 = code byte index, head = kb; accumulator p = bit position
    const float inv_fv = ldexpf(1.f, -Fv);
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const float v = fmaf(fmaf(fmaf((float)acc[p][3], 256.f, (float)acc[p][2]), 256.f,
                                (float)acc[p][1]), 256.f, (float)acc[p][0]);
      const int ch = 32 * (n16 >> 2) + 31 - 8 * (n16 & 3) - p;
      const float w = ldexpf(inv_fv, -p) * (p == 7 ? -1.f : 1.f);
      partial[kb * kD + ch] = v * w;
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int h = 0; h < kHeads; ++h) {
    if (kb == 0) {
#pragma unroll
      for (int c = 0; c < 8; ++c) partial[h * kD + 8 * n16 + c] += tacc[h][c];
    }
    const float l = wave_sum(lsum[h] + tl[h]);
    const float m = wave_sum(msum[h]);
    if (lane == 0) {
      red[(wave * kHeads + h) * 6 + 3] = l;
      red[(wave * kHeads + h) * 6 + 4] = m;
    }
  }
  __syncthreads();

  CQ_CLK(10);
  // ---- epilogue: sum the waves, add the additive value term, normalise, round to fp16
  {
    const int h = tid / kD, c = tid % kD;
    if (h < a.g) {
      float num = 0.f, l = 0.f, m = 0.f;
      for (int w = 0; w < kWaves; ++w) {
        num += reinterpret_cast<float*>(smem)[((size_t)w * kHeads + h) * kD + c];
        l += red[(w * kHeads + h) * 6 + 3];
        m += red[(w * kHeads + h) * 6 + 4];
      }
      a.out[((size_t)b * a.Hq + (size_t)kvh * a.g + h) * kD + c] = __float2half_rn((num + m) / l);
    }
  }
  (void)n_all;
  CQ_CLK(11);
}

}  // namespace

#ifdef CQ_PHASE_CLOCKS
static long long* g_phase_clocks = nullptr;
extern "C" void cq_debug_set_phase_clocks(void* p) { g_phase_clocks = static_cast<long long*>(p); }
#endif

size_t fused_lds_bytes(int g, int n_vis, int n_text, int k_group, int* stride_out) {
  int stride = n_vis + n_text;
  stride += (16 - (stride % 32) + 32) % 32;      // stride = 16 (mod 32): conflict-free head rows
  if (stride_out) *stride_out = stride;
  size_t off = (size_t)kHeads * stride * sizeof(float);
  const size_t part = (size_t)kWaves * kHeads * kD * sizeof(float);
  if (off < part) off = part;
  off += kHeads * kD * sizeof(float);
  const int n_groups = k_group > 0 ? n_vis / k_group : 0;
  off += (size_t)kHeads * (n_groups > 0 ? n_groups : 1) * sizeof(float);
  off = (off + 15) & ~(size_t)15;
  off += (size_t)kWaves * kStageBytes;
  off += (size_t)kWaves * kHeads * 6 * sizeof(float);
  (void)g;
  return off;
}

bool fused_supported(const DecodeShape& s) {
  if (s.d != kD || s.bits != 1) return false;
  if (s.k_axis != CQ_AXIS_CHANNEL || s.v_axis != CQ_AXIS_TOKEN || s.v_group != kD) return false;
  if ((s.k_group != 32 && s.k_group != 64 && s.k_group != 128) || s.g > kHeads) return false;
  if (s.n_vis > 65536 || s.n_vis % 64 != 0) return false;
  return fused_lds_bytes(s.g, s.n_vis, s.n_text, s.k_group, nullptr) <= 160 * 1024;
}

hipError_t launch_decode_fused(const DecodeShape& s, const void* q, const cq_qtensor_t& k,
                               const cq_qtensor_t& v, const void* k_text, const void* v_text,
                               const Calib& calib, float softmax_scale, void* out,
                               hipStream_t stream) {
  FusedArgs a;
  a.q = static_cast<const __half*>(q);
  a.k_codes = k.codes; a.k_scale = k.scale; a.k_min = k.min;
  a.v_codes = v.codes; a.v_scale = v.scale; a.v_min = v.min;
  a.k_text = static_cast<const __half*>(k_text);
  a.v_text = static_cast<const __half*>(v_text);
  a.out = static_cast<__half*>(out);
  a.Hq = s.Hq; a.Hkv = s.Hkv; a.g = s.g; a.n_vis = s.n_vis; a.n_text = s.n_text;
  a.n_text_cap = s.n_text_cap; a.k_group = s.k_group;
  a.calib_mode = calib.mode; a.tau1 = calib.tau1; a.tau2 = calib.tau2;
  a.gamma = calib.gamma; a.delta = calib.delta; a.softmax_scale = softmax_scale;
#ifdef CQ_PHASE_CLOCKS
  a.clocks = g_phase_clocks;
#endif
  const size_t lds = fused_lds_bytes(s.g, s.n_vis, s.n_text, s.k_group, &a.stride);
  void (*kern)(const FusedArgs) = nullptr;
  int slot = 0;
  switch (s.k_group) {
    case 32: kern = fused_row_kernel<2>; slot = 0; break;
    case 64: kern = fused_row_kernel<4>; slot = 1; break;
    case 128: kern = fused_row_kernel<8>; slot = 2; break;
    default: return hipErrorInvalidValue;
  }
  static size_t configured[3] = {0, 0, 0};
  if (lds > configured[slot]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured[slot] = lds;
  }
  kern<<<dim3(s.B * s.Hkv), dim3(kThreads), lds, stream>>>(a);
  return hipGetLastError();
}

}  // namespace cq
