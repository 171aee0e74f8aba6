// CPU oracle for CalibQuant's hot path (arxiv 2502.14882), C++ twin: TEST INFRASTRUCTURE ONLY.
//
// The same plain fp64 statement of the method as oracle/cq_oracle.py (the numpy oracle), written
// a second time so that (i) whole benchmark-size calls can be checked row by row and timed on all
// host cores, and (ii) the two oracles can be checked against each other (codes and stored
// parameters bit for bit, attention to 1e-12).  It follows the paper's steps in the paper's order
// with no blocking, fusion or rearrangement: quantize -> pack -> unpack -> dequantize ->
// q K_deq^T -> g on the visual logits -> joint softmax -> weights times [V_deq; V_text].  In
// particular the logits are formed on the DEQUANTIZED keys (Sec. 2.1 on the output of the Sec. 2.2
// dequantize equation), not by the post-scaling rearrangement of Sec. 3.1.
// It shares nothing with the HIP kernels (no header, table, constant or helper) and is never
// called by the product path; only tests, the smoke check and the benchmark's cpu_baseline leg
// load it.  OpenMP spreads independent (batch, KV head) rows over the host's threads; inside a
// row everything is a sequential loop.
//
// What each function follows
//   half_to_double            IEEE 754 binary16 (the cache's and the query's storage type)
//   cqo_quantize              Sec. 3.1 alpha/beta per group, Sec. 2.2 quantize equation, the stored
//                             "scale factor and bias term" of Sec. 3.1, appendix pack(v, N, M = 32)
//   unpack_code               appendix unpack(u, N, M)
//   dequantize_row            Sec. 2.2 dequantize equation with the stored parameters
//   cqo_decode_attn           Sec. 2.1 softmax(q K^T / sqrt(d)) V on the dequantized cache, with
//                             Sec. 3.2's g on the visual logits and the 16-bit text tail of Sec. 3
// Readings of the silent points are those listed in the numpy oracle's header (R1-R6): exact
// rounding with ties to even, statistics per group, min as fp16 / scale rounded once to float32,
// 32-bit words with the first element in the top bits, gamma/delta = extrema of a row's visual
// logits after scaling, query head hq reads KV head hq / (Hq / Hkv).
// parity unpinned: as in the numpy oracle (tau values, value axis, group sizes, fp32 scale).
#include <cfenv>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { AXIS_CHANNEL = 0, AXIS_TOKEN = 1 };
enum { CALIB_NONE = 0, CALIB_DYNAMIC = 1, CALIB_FIXED = 2 };

// binary16 -> double, exact (sign, 5 exponent bits, 10 fraction bits; subnormals; no Inf/NaN inputs)
double half_to_double(uint16_t h) {
  const int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
  double v;
  if (e == 0) v = std::ldexp((double)f, -24);                 // subnormal or zero
  else if (e == 31) v = f ? NAN : INFINITY;
  else v = std::ldexp((double)(1024 + f), e - 25);
  return sign ? -v : v;
}

// double -> binary16 bits for a value that IS a binary16 number (the group minimum is an input
// element); a zero of either sign is stored as +0
uint16_t exact_double_to_half(double v) {
  if (v == 0.0) return 0;
  const uint16_t sign = v < 0 ? 0x8000 : 0;
  double a = std::fabs(v);
  int e;
  const double m = std::frexp(a, &e);          // a = m * 2^e, m in [0.5, 1)
  if (e - 1 < -14) {                           // subnormal: a = f * 2^-24
    return sign | (uint16_t)std::ldexp(a, 24);
  }
  const int f = (int)std::ldexp(m, 11) - 1024; // 11 significant bits
  return sign | (uint16_t)(((e - 1 + 15) << 10) | f);
}

// element i of a 32-bit word holding N-bit codes: (u >> (32 - N(1 + i))) mod 2^N   (appendix unpack)
inline unsigned unpack_code(const uint32_t* words, int c, int bits) {
  const int per = 32 / bits;
  return (words[c / per] >> (32 - bits * (1 + c % per))) & ((1u << bits) - 1u);
}

// x_deq = x_dis * scale + min with the STORED parameters, one [n, d] row of a tensor, fp64
void dequantize_row(const uint32_t* words, const float* scale, const uint16_t* minv, int n, int d,
                    int bits, int axis, int group, double* out) {
  const int wpt = d * bits / 32;
  for (int j = 0; j < n; ++j)
    for (int c = 0; c < d; ++c) {
      const size_t meta = axis == AXIS_CHANNEL ? (size_t)(j / group) * d + c
                                               : (size_t)j * (d / group) + c / group;
      const double code = (double)unpack_code(words + (size_t)j * wpt, c, bits);
      out[(size_t)j * d + c] = code * (double)scale[meta] + half_to_double(minv[meta]);
    }
}

}  // namespace

extern "C" {

// threads the parallel loops below will use
int cqo_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// Quantize `rows` independent [n, d] fp16 matrices (Sec. 2.2 + Sec. 3.1 + appendix).
//   x_f16   [rows][n][d] binary16 bits
//   words   [rows][n][d*bits/32]; scale, minv: [rows][n/group][d] (AXIS_CHANNEL) or
//           [rows][n][d/group] (AXIS_TOKEN)
// Returns 0, or -1 for sizes that do not divide.
int cqo_quantize(const uint16_t* x_f16, int64_t rows, int n, int d, int bits, int axis, int group,
                 uint32_t* words, float* scale, uint16_t* minv) {
  if (bits < 1 || bits > 8 || 32 % bits != 0 || (d * bits) % 32 != 0 || group < 1) return -1;
  if (axis == AXIS_CHANNEL ? n % group != 0 : d % group != 0) return -1;
  if (std::fegetround() != FE_TONEAREST) return -2;      // nearbyint below must round to even
  const double L = (double)((1 << bits) - 1);
  const int wpt = d * bits / 32, per = 32 / bits;
  const size_t meta_per_row = axis == AXIS_CHANNEL ? (size_t)(n / group) * d : (size_t)n * (d / group);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t r = 0; r < rows; ++r) {
    const uint16_t* x = x_f16 + (size_t)r * n * d;
    uint32_t* w = words + (size_t)r * n * wpt;
    float* sc = scale + (size_t)r * meta_per_row;
    uint16_t* mn = minv + (size_t)r * meta_per_row;
    std::memset(w, 0, (size_t)n * wpt * sizeof(uint32_t));
    const int n_groups = axis == AXIS_CHANNEL ? (n / group) * d : n * (d / group);
    for (int gi = 0; gi < n_groups; ++gi) {
      // the elements of group gi: (token j0 + i * tj, channel c0 + i * tc), i < group
      int j0, c0, tj, tc;
      if (axis == AXIS_CHANNEL) { j0 = (gi / d) * group; c0 = gi % d; tj = 1; tc = 0; }
      else { j0 = gi / (d / group); c0 = (gi % (d / group)) * group; tj = 0; tc = 1; }
      // alpha = min, beta = max over the group (Sec. 3.1)
      double alpha = INFINITY, beta = -INFINITY;
      for (int i = 0; i < group; ++i) {
        const double v = half_to_double(x[(size_t)(j0 + i * tj) * d + c0 + i * tc]);
        if (v < alpha) alpha = v;
        if (v > beta) beta = v;
      }
      const double D = beta - alpha;                       // exact in fp64 for binary16 inputs
      sc[gi] = (float)(D / L);                             // one rounding to float32
      mn[gi] = exact_double_to_half(alpha);
      for (int i = 0; i < group; ++i) {
        const int j = j0 + i * tj, c = c0 + i * tc;
        const double v = half_to_double(x[(size_t)j * d + c]);
        // x_dis = round((x - alpha)(2^b - 1) / (beta - alpha)), ties to even; constant group -> 0
        const unsigned code = D > 0.0 ? (unsigned)std::nearbyint((v - alpha) * L / D) : 0u;
        // pack: code i of a word shifted left by 32 - N(1 + i), summed (appendix)
        w[(size_t)j * wpt + c / per] += code << (32 - bits * (1 + c % per));
      }
    }
  }
  return 0;
}

// One decode step over a quantized visual cache plus a 16-bit text tail (Sec. 2.1, 3.2, 3).
//   q_f16 [B][Hq][d]; k_*/v_*: one quantized tensor each for [B][Hkv][n_vis][d] as written by
//   cqo_quantize; k_text_f16 / v_text_f16 [B][Hkv][n_text_cap][d] (first n_text tokens attended);
//   out [B][Hq][d] fp64.  softmax_scale 0 means 1/sqrt(d).  Returns 0, or -1 for bad sizes.
int cqo_decode_attn(const uint16_t* q_f16, const uint32_t* k_words, const float* k_scale,
                    const uint16_t* k_min, int k_axis, int k_group, const uint32_t* v_words,
                    const float* v_scale, const uint16_t* v_min, int v_axis, int v_group,
                    const uint16_t* k_text_f16, const uint16_t* v_text_f16, int B, int Hq, int Hkv,
                    int d, int n_vis, int bits, int n_text, int n_text_cap, int calib_mode,
                    double tau1, double tau2, double gamma, double delta, double softmax_scale,
                    double* out) {
  if (B < 1 || Hkv < 1 || Hq % Hkv != 0 || n_text > n_text_cap || n_vis + n_text < 1) return -1;
  if (n_vis > 0 && (k_group < 1 || v_group < 1)) return -1;
  const int g = Hq / Hkv, wpt = d * bits / 32;
  if (softmax_scale == 0.0) softmax_scale = 1.0 / std::sqrt((double)d);
  const size_t k_meta = n_vis == 0 ? 0 : (k_axis == AXIS_CHANNEL ? (size_t)(n_vis / k_group) * d : (size_t)n_vis * (d / k_group));
  const size_t v_meta = n_vis == 0 ? 0 : (v_axis == AXIS_CHANNEL ? (size_t)(n_vis / v_group) * d : (size_t)n_vis * (d / v_group));
#pragma omp parallel
  {
    std::vector<double> k_deq((size_t)n_vis * d), v_deq((size_t)n_vis * d);
    std::vector<double> s((size_t)n_vis + n_text), qd(d);
#pragma omp for schedule(dynamic, 1)
    for (int r = 0; r < B * Hkv; ++r) {
      // dequantize the row's keys and values (Sec. 2.2)
      if (n_vis > 0) {
        dequantize_row(k_words + (size_t)r * n_vis * wpt, k_scale + (size_t)r * k_meta,
                       k_min + (size_t)r * k_meta, n_vis, d, bits, k_axis, k_group, k_deq.data());
        dequantize_row(v_words + (size_t)r * n_vis * wpt, v_scale + (size_t)r * v_meta,
                       v_min + (size_t)r * v_meta, n_vis, d, bits, v_axis, v_group, v_deq.data());
      }
      const uint16_t* kt = k_text_f16 ? k_text_f16 + (size_t)r * n_text_cap * d : nullptr;
      const uint16_t* vt = v_text_f16 ? v_text_f16 + (size_t)r * n_text_cap * d : nullptr;
      const int b = r / Hkv, h = r % Hkv;
      for (int hg = 0; hg < g; ++hg) {
        const size_t hq = (size_t)b * Hq + (size_t)h * g + hg;
        for (int c = 0; c < d; ++c) qd[c] = half_to_double(q_f16[hq * d + c]);
        // logits q K_deq^T / sqrt(d) on the visual tokens (Sec. 2.1)
        double lo = INFINITY, hi = -INFINITY;
        for (int j = 0; j < n_vis; ++j) {
          double acc = 0.0;
          for (int c = 0; c < d; ++c) acc += qd[c] * k_deq[(size_t)j * d + c];
          s[j] = acc * softmax_scale;
          if (s[j] < lo) lo = s[j];
          if (s[j] > hi) hi = s[j];
        }
        // g(x) = (delta - gamma + tau1 - tau2)/(delta - gamma) (x - gamma) + gamma - tau1 on the
        // visual logits only (Sec. 3.2); delta == gamma -> slope 1
        if (calib_mode != CALIB_NONE && n_vis > 0) {
          const double gam = calib_mode == CALIB_DYNAMIC ? lo : gamma;
          const double del = calib_mode == CALIB_DYNAMIC ? hi : delta;
          const double width = del - gam;
          const double slope = width == 0.0 ? 1.0 : (width + tau1 - tau2) / width;
          for (int j = 0; j < n_vis; ++j) s[j] = slope * (s[j] - gam) + gam - tau1;
        }
        // text logits, not calibrated (Sec. 3: only the visual tokens are quantized)
        for (int t = 0; t < n_text; ++t) {
          double acc = 0.0;
          for (int c = 0; c < d; ++c) acc += qd[c] * half_to_double(kt[(size_t)t * d + c]);
          s[n_vis + t] = acc * softmax_scale;
        }
        // joint softmax and the weighted value sum (Sec. 2.1)
        const int n_all = n_vis + n_text;
        double m = -INFINITY, den = 0.0;
        for (int j = 0; j < n_all; ++j) if (s[j] > m) m = s[j];
        for (int j = 0; j < n_all; ++j) { s[j] = std::exp(s[j] - m); den += s[j]; }
        double* o = out + hq * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int j = 0; j < n_vis; ++j) {
          const double w = s[j] / den;
          for (int c = 0; c < d; ++c) o[c] += w * v_deq[(size_t)j * d + c];
        }
        for (int t = 0; t < n_text; ++t) {
          const double w = s[n_vis + t] / den;
          for (int c = 0; c < d; ++c) o[c] += w * half_to_double(vt[(size_t)t * d + c]);
        }
      }
    }
  }
  return 0;
}

}  // extern "C"
