// Tuned quantizer for head_dim 128, b in {1, 2, 4, 8}, groups of 32/64/128 or, channel-wise, the
// whole sequence (gfx950).
//
// One 256-thread block quantizes a tile of 128 tokens x 128 channels (32 KB of fp16), read once
// with 16-byte loads and kept in registers:
//   lane = (token slot lane/16, channel octet lane%16); wave w owns tokens 32w .. 32w+31, so a
//   wave-wide load is 4 whole token rows = 1 KB contiguous.
//   1. min/max of Sec. 3.1 with packed-half min/max: over tokens (channel axis: in-thread, then
//      across the 4 token slots and, for groups > 32 tokens, across waves through LDS) or over
//      channels (token axis: in-thread over the octet, then across the lanes of a channel group).
//   2. one thread per (group, channel) resp. (token, channel group) derives, in fp64 where every
//      quantity is exact, the stored scale/min and 2^b-1 fp16 thresholds t_k such that for every
//      fp16 x:  x > t_k  <=>  round-half-even((x-min)(2^b-1)/(max-min)) >= k   (Sec. 2.2 equation).
//   3. codes by comparing packed halves against the thresholds (sign of t - x), bits gathered with
//      v_perm + v_dot4, words assembled across adjacent lanes, MSB first as in the packing appendix.
//   b in {4, 8} (too many thresholds): step 2 stores min and (2^b-1)/(max-min) per group, step 3
//   evaluates the quantize equation per element with that reciprocal - in fp32 where that already
//   decides the code, in fp64 with the rounding settled exactly (see exact_code) where it does
//   not; a lane's 8 channels fill one word (b = 4) or two (b = 8).
// Channel-wise statistics over the whole sequence (group = n_vis: one pair per channel, Sec. 3.1
// as printed) take a pass of their own: row_extrema_kernel leaves kSplits partial (min, max)
// pairs per channel in the code words of the row's LAST tile (the caller's output buffer: no
// other memory is needed), the tile kernel reduces them instead of computing tile statistics,
// and the last tile of every row is quantized by a second launch, after all other tiles have
// read the partials it overwrites.
// Results are bit-identical to evaluating the quantize equation element by element in fp64.
#include <hip/hip_fp16.h>

#include "cq_internal.h"

namespace cq {
namespace {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kTile = 128;       // tokens per block
constexpr int kThreads = 256;
constexpr int kSplits = 4;       // partial extrema per row: 4 x 128 x (min, max) fp16 = 2 KB = one tile's
                                 // code words at b = 1

// ---- fp16 bit patterns as an ordered set
__device__ inline uint16_t h_key(uint16_t u) { return (u & 0x8000u) ? (uint16_t)~u : (uint16_t)(u | 0x8000u); }
__device__ inline uint16_t h_unkey(uint16_t k) { return (k & 0x8000u) ? (uint16_t)(k & 0x7fffu) : (uint16_t)~k; }
__device__ inline uint16_t h_next(uint16_t u) { return h_unkey((uint16_t)(h_key(u) + 1)); }
__device__ inline uint16_t h_prev(uint16_t u) { return h_unkey((uint16_t)(h_key(u) - 1)); }
__device__ inline double h_to_double(uint16_t u) { return (double)__half2float(__ushort_as_half(u)); }

// Largest fp16 t (as bits) with  NOT [ 2L(t - alpha) ? (2k-1) D ],  ? being > for odd k and >= for
// even k (the even side of a tie).  Then code >= k  <=>  x > t for every fp16 x.
__device__ inline uint16_t threshold_bits(double alpha, double D, int k, int L) {
  if (!(D > 0.0)) return 0x7bffu;            // constant group: nothing exceeds the largest finite
  const double rhs = (double)(2 * k - 1) * D, twoL = 2.0 * L;
  const bool strict = (k & 1) != 0;
  auto pred = [&](uint16_t u) {
    const double lhs = twoL * (h_to_double(u) - alpha);
    return strict ? lhs > rhs : lhs >= rhs;
  };
  // candidate: the real-valued boundary, good to an fp16 step (the reciprocal of 2L is a compile-time
  // constant at every call site; the loops below make the result exact whatever the candidate)
  uint16_t t = __half_as_ushort(__float2half_rn((float)(alpha + rhs * (1.0 / twoL))));
  for (int it = 0; it < 4 && pred(t); ++it) t = h_prev(t);
  for (int it = 0; it < 4 && !pred(h_next(t)); ++it) t = h_next(t);
  return t == 0x8000u ? (uint16_t)0 : t;     // -0 would break the sign test against +0
}

__device__ inline uint16_t canonical_zero(uint16_t bits) { return (bits & 0x7fffu) == 0 ? (uint16_t)0 : bits; }

// sign bits of (t - x) for 8 channels -> 0x80 per channel, channels 0..3 in xa, 4..7 in xb
__device__ inline void sign_bytes(const v8h& t, const v8h& x, uint32_t& xa, uint32_t& xb) {
  const v8h d = t - x;
  const v4u u = __builtin_bit_cast(v4u, d);
  xa = __builtin_amdgcn_perm(u[1], u[0], 0x07050301u) & 0x80808080u;
  xb = __builtin_amdgcn_perm(u[3], u[2], 0x07050301u) & 0x80808080u;
}

// code bits of one octet of one token: 8 bits (b = 1) or 16 bits (b = 2), first channel highest
template <int BITS>
__device__ inline uint32_t octet_codes(const v8h& x, const v8h* thr) {
  if constexpr (BITS == 1) {
    uint32_t xa, xb;
    sign_bytes(thr[0], x, xa, xb);
    const uint32_t s = __builtin_amdgcn_udot4(xa, 0x10204080u, 0u, false);
    return __builtin_amdgcn_udot4(xb, 0x01020408u, s, false) >> 7;
  } else {
    uint32_t a1, b1, a2, b2, a3, b3;
    sign_bytes(thr[0], x, a1, b1);
    sign_bytes(thr[1], x, a2, b2);
    sign_bytes(thr[2], x, a3, b3);
    const uint32_t la = a1 ^ a2 ^ a3, lb = b1 ^ b2 ^ b3;     // low code bit; high bit is [x > t2]
    uint32_t up = __builtin_amdgcn_udot4(a2, 0x02082080u, 0u, false);
    up = __builtin_amdgcn_udot4(la, 0x01041040u, up, false);
    uint32_t lo = __builtin_amdgcn_udot4(b2, 0x02082080u, 0u, false);
    lo = __builtin_amdgcn_udot4(lb, 0x01041040u, lo, false);
    return ((up >> 7) << 8) | (lo >> 7);
  }
}

// round-half-even((x - alpha) L / D) for b in {4, 8}, from rinv = fl(L / D) (0 for a constant group).
// x - alpha is exact in fp64; q = fl((x - alpha) * rinv) is within 2^-44 of the true quotient
// (two roundings, q <= 255).  The true quotient is a ratio of integers with denominator
// D / 2^-24 < 2^41, so it is either exactly k + 1/2 or at least 2^-42 away from it: a computed
// fraction within 2^-43 of 1/2 is a tie (to even), anything else rounds by its computed fraction.
__device__ inline uint32_t exact_code(_Float16 x, double alpha, double rinv) {
  const double q = ((double)(float)x - alpha) * rinv;
  const double f = floor(q);
  const double frac = q - f;
  uint32_t c = (uint32_t)(int)f;
  if (fabs(frac - 0.5) < 0x1p-43) c += c & 1u;
  else c += frac > 0.5 ? 1u : 0u;
  return c;
}

// the 8 codes of one octet as packed words, first channel in the top bits (packing appendix).
// Fast path in fp32 with alpha32 = alpha and rinv32 = fl32(rinv): q32 = fl(fl(x - alpha) * rinv32)
// carries three roundings, so it is within L * 3 * 2^-24 of the true quotient (L = 2^b - 1 bounds
// the quotient).  Unless q32 lies within L * 2^-22 of a half-integer, rounding it to nearest gives
// the exact code; an octet with any element inside that band (8-bit codes: ~0.1 % of the octets)
// is redone by exact_code.
template <int BITS>
__device__ inline void octet_words(const v8h& x, const double (&alpha)[8], const double (&rinv)[8],
                                   const float (&alpha32)[8], const float (&rinv32)[8],
                                   uint32_t& w0, uint32_t& w1) {
  constexpr float kBand = (float)((1 << BITS) - 1) * 0x1p-22f;
  uint32_t c[8];
  bool unsure = false;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float q = ((float)x[j] - alpha32[j]) * rinv32[j];
    const float r = rintf(q);
    c[j] = (uint32_t)(int)r;
    unsure |= 0.5f - fabsf(q - r) <= kBand;
  }
  if (unsure) {
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = exact_code(x[j], alpha[j], rinv[j]);
  }
  if constexpr (BITS == 4) {
    w0 = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) w0 |= c[j] << (28 - 4 * j);
    w1 = 0;
  } else {
    w0 = (c[0] << 24) | (c[1] << 16) | (c[2] << 8) | c[3];
    w1 = (c[4] << 24) | (c[5] << 16) | (c[6] << 8) | c[7];
  }
}

struct QArgs {
  const __half* x;
  uint32_t* codes;
  float* scale;
  uint16_t* minv;
  // whole-sequence statistics only: tiles per row, and the tiles of every row that this launch
  // covers (tile_first .. tile_first + tiles_launch - 1)
  int tiles_row, tile_first, tiles_launch;
  unsigned launch_magic;   // fl(2^32 / tiles_launch) + 1 if exact for every block of the launch, else 0
};

// Partial extrema of a row's split sp live at [(sp * 2 + {0: min, 1: max}) * kD + channel], fp16,
// in the code words of the row's last tile.
__device__ inline _Float16* row_partials(const QArgs& a, int row, int words_per_token) {
  const size_t last_tok = ((size_t)row * a.tiles_row + (a.tiles_row - 1)) * kTile;
  return reinterpret_cast<_Float16*>(a.codes + last_tok * words_per_token);
}

// First pass of whole-sequence statistics: block (row, sp) scans its share of the row's tiles.
template <int BITS>
__global__ void __launch_bounds__(kThreads)
row_extrema_kernel(const QArgs a) {
  __shared__ __align__(16) _Float16 s_part[2][4][kD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c8 = lane & 15, ts = lane >> 4;
  const int row = blockIdx.x / kSplits, sp = blockIdx.x % kSplits;
  const int ta = a.tiles_row * sp / kSplits, tb = a.tiles_row * (sp + 1) / kSplits;
  const v8h* src = reinterpret_cast<const v8h*>(a.x) +
                   ((size_t)row * a.tiles_row * kTile + 32 * wave + ts) * (kD / 8) + c8;
  const _Float16 inf = __builtin_bit_cast(_Float16, (uint16_t)0x7c00u);
  v8h mn = {inf, inf, inf, inf, inf, inf, inf, inf};        // an empty share leaves the neutral pair
  v8h mx = -mn;
  for (int t = ta; t < tb; ++t) {
    v8h x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = src[((size_t)t * kTile + 4 * i) * (kD / 8)];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      mn = __builtin_elementwise_min(mn, x[i]);
      mx = __builtin_elementwise_max(mx, x[i]);
    }
  }
  v4u mnu = __builtin_bit_cast(v4u, mn), mxu = __builtin_bit_cast(v4u, mx);
#pragma unroll
  for (int o = 16; o <= 32; o <<= 1) {
    v4u on, ox;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      on[r] = __shfl_xor(mnu[r], o);
      ox[r] = __shfl_xor(mxu[r], o);
    }
    mn = __builtin_elementwise_min(mn, __builtin_bit_cast(v8h, on));
    mx = __builtin_elementwise_max(mx, __builtin_bit_cast(v8h, ox));
    mnu = __builtin_bit_cast(v4u, mn);
    mxu = __builtin_bit_cast(v4u, mx);
  }
  if (ts == 0) {
    *reinterpret_cast<v8h*>(&s_part[0][wave][c8 * 8]) = mn;
    *reinterpret_cast<v8h*>(&s_part[1][wave][c8 * 8]) = mx;
  }
  __syncthreads();
  if (tid < kD) {
    _Float16 lo = s_part[0][0][tid], hi = s_part[1][0][tid];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      lo = (_Float16)fminf((float)lo, (float)s_part[0][w][tid]);
      hi = (_Float16)fmaxf((float)hi, (float)s_part[1][w][tid]);
    }
    _Float16* part = row_partials(a, row, kD * BITS / 32);
    part[(sp * 2 + 0) * kD + tid] = lo;
    part[(sp * 2 + 1) * kD + tid] = hi;
  }
}

// AXIS: CQ_AXIS_CHANNEL (GROUP tokens per group; GROUP = 0: the whole sequence, extrema from
// row_extrema_kernel) or CQ_AXIS_TOKEN (GROUP channels per group)
template <int AXIS, int BITS, int GROUP>
__global__ void __launch_bounds__(kThreads)
quantize_tile_kernel(const QArgs a) {
  constexpr int L = (1 << BITS) - 1;
  constexpr int kWords = kD * BITS / 32;                  // words per token
  constexpr bool kWhole = GROUP == 0;
  static_assert(!kWhole || AXIS == CQ_AXIS_CHANNEL, "whole-sequence statistics are channel-wise");
  constexpr int kG = kWhole ? kTile : GROUP;              // a tile of a whole row is one group
  constexpr int NG = AXIS == CQ_AXIS_CHANNEL ? kTile / kG : kD / kG;         // groups per tile / token
  __shared__ __align__(16) _Float16 s_part[2][4][kD];     // channel axis: per-wave min, max
  __shared__ __align__(16) _Float16 s_stat[kTile][4][2];  // token axis: min, max per (token, group)
  constexpr bool kWide = BITS > 2;                        // per-element arithmetic instead of thresholds
  __shared__ __align__(16) _Float16 s_thr[kWide ? 8 : (AXIS == CQ_AXIS_CHANNEL ? NG * L * kD : kTile * 4 * 4)];
  __shared__ __align__(16) double s_rinv[kWide ? (AXIS == CQ_AXIS_CHANNEL ? NG * kD : kTile * 4) : 1];
  __shared__ __align__(16) _Float16 s_alpha[kWide ? (AXIS == CQ_AXIS_CHANNEL ? NG * kD : kTile * 4) : 8];
  __shared__ __align__(16) uint32_t s_codes[kTile * kWords];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c8 = lane & 15, ts = lane >> 4;
  // tiles never straddle rows (n_vis % 128 == 0)
  // block = row * tiles_launch + tile; the quotient by the host's fl(2^32 / tiles_launch) + 1 where
  // that is exact (a division by a run-time value costs dozens of instructions ahead of the loads)
  int wrow = 0, wtile = 0;
  if constexpr (kWhole) {
    wrow = a.tiles_launch == 1 ? (int)blockIdx.x
         : a.launch_magic ? (int)__umulhi(blockIdx.x, a.launch_magic) : (int)(blockIdx.x / (unsigned)a.tiles_launch);
    wtile = a.tile_first + (int)blockIdx.x - wrow * a.tiles_launch;
  }
  const size_t tok0 = kWhole ? ((size_t)wrow * a.tiles_row + wtile) * kTile : (size_t)blockIdx.x * kTile;
  const v8h* src = reinterpret_cast<const v8h*>(a.x) + (tok0 + 32 * wave + ts) * (kD / 8) + c8;

  v8h x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)                                              // token 32w + 4i + ts
    x[i] = __builtin_nontemporal_load(src + (size_t)i * 4 * (kD / 8));   // read exactly once

  if constexpr (kWhole) {
    // ---- 1 + 2. the row's extrema from the partials of the first pass; parameters and thresholds
    if (tid < kD) {
      const int c = tid;
      const _Float16* part = row_partials(a, wrow, kWords);
      _Float16 lo = part[c], hi = part[kD + c];
#pragma unroll
      for (int sp = 1; sp < kSplits; ++sp) {
        lo = (_Float16)fminf((float)lo, (float)part[(sp * 2 + 0) * kD + c]);
        hi = (_Float16)fmaxf((float)hi, (float)part[(sp * 2 + 1) * kD + c]);
      }
      const uint16_t mbits = canonical_zero(__builtin_bit_cast(uint16_t, lo));
      const double alpha = h_to_double(mbits);
      const double D = ((double)(float)hi - alpha) + 0.0;
      if (wtile == a.tiles_row - 1) {          // one block per row stores the parameters
        a.scale[(size_t)wrow * kD + c] = (float)(D / (double)L);
        a.minv[(size_t)wrow * kD + c] = mbits;
      }
      if constexpr (kWide) {
        s_alpha[c] = __builtin_bit_cast(_Float16, mbits);
        s_rinv[c] = D > 0.0 ? (double)L / D : 0.0;
      } else {
#pragma unroll
        for (int k = 1; k <= L; ++k)
          s_thr[(k - 1) * kD + c] = __builtin_bit_cast(_Float16, threshold_bits(alpha, D, k, L));
      }
    }
    __syncthreads();   // in the row's last tile this also orders the reads above before the
                       // block's own code words, which replace the partials
  } else if constexpr (AXIS == CQ_AXIS_CHANNEL) {
    // ---- 1. per-channel extrema over the wave's 32 tokens
    v8h mn = x[0], mx = x[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
      mn = __builtin_elementwise_min(mn, x[i]);
      mx = __builtin_elementwise_max(mx, x[i]);
    }
    v4u mnu = __builtin_bit_cast(v4u, mn), mxu = __builtin_bit_cast(v4u, mx);
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
      v4u on, ox;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        on[r] = __shfl_xor(mnu[r], o);
        ox[r] = __shfl_xor(mxu[r], o);
      }
      mn = __builtin_elementwise_min(mn, __builtin_bit_cast(v8h, on));
      mx = __builtin_elementwise_max(mx, __builtin_bit_cast(v8h, ox));
      mnu = __builtin_bit_cast(v4u, mn);
      mxu = __builtin_bit_cast(v4u, mx);
    }
    if (ts == 0) {
      *reinterpret_cast<v8h*>(&s_part[0][wave][c8 * 8]) = mn;
      *reinterpret_cast<v8h*>(&s_part[1][wave][c8 * 8]) = mx;
    }
    __syncthreads();
    // ---- 2. one thread per (group, channel): stored parameters and thresholds
    constexpr int kWavesPerGroup = GROUP / 32;
    for (int item = tid; item < NG * kD; item += kThreads) {
      const int g = item / kD, c = item % kD;
      _Float16 lo = s_part[0][g * kWavesPerGroup][c], hi = s_part[1][g * kWavesPerGroup][c];
#pragma unroll
      for (int w = 1; w < kWavesPerGroup; ++w) {
        lo = (_Float16)fminf((float)lo, (float)s_part[0][g * kWavesPerGroup + w][c]);
        hi = (_Float16)fmaxf((float)hi, (float)s_part[1][g * kWavesPerGroup + w][c]);
      }
      const uint16_t mbits = canonical_zero(__builtin_bit_cast(uint16_t, lo));
      const double alpha = h_to_double(mbits);
      const double D = ((double)(float)hi - alpha) + 0.0;
      const size_t meta = (tok0 / GROUP + g) * kD + c;
      a.scale[meta] = (float)(D / (double)L);
      a.minv[meta] = mbits;
      if constexpr (kWide) {
        s_alpha[g * kD + c] = __builtin_bit_cast(_Float16, mbits);
        s_rinv[g * kD + c] = D > 0.0 ? (double)L / D : 0.0;
      } else {
#pragma unroll
        for (int k = 1; k <= L; ++k)
          s_thr[(g * L + (k - 1)) * kD + c] =
              __builtin_bit_cast(_Float16, threshold_bits(alpha, D, k, L));
      }
    }
    __syncthreads();
  }
  if constexpr (AXIS == CQ_AXIS_CHANNEL) {
    // ---- 3. codes
    const int g = (32 * wave) / kG;
    if constexpr (kWide) {
      double al[8], ri[8];
      float al32[8], ri32[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        al32[j] = (float)s_alpha[g * kD + c8 * 8 + j];
        al[j] = (double)al32[j];
        ri[j] = s_rinv[g * kD + c8 * 8 + j];
        ri32[j] = (float)ri[j];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int tok = 32 * wave + 4 * i + ts;
        uint32_t w0, w1;
        octet_words<BITS>(x[i], al, ri, al32, ri32, w0, w1);
        if constexpr (BITS == 4) {
          s_codes[tok * kWords + c8] = w0;
        } else {
          s_codes[tok * kWords + 2 * c8] = w0;
          s_codes[tok * kWords + 2 * c8 + 1] = w1;
        }
      }
    } else {
    v8h thr[L];
#pragma unroll
    for (int k = 0; k < L; ++k) thr[k] = *reinterpret_cast<const v8h*>(&s_thr[(g * L + k) * kD + c8 * 8]);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      uint32_t bits = octet_codes<BITS>(x[i], thr);
      const int tok = 32 * wave + 4 * i + ts;
      if constexpr (BITS == 1) {
        bits <<= 24 - 8 * (c8 & 3);
        bits |= __shfl_xor(bits, 1);
        bits |= __shfl_xor(bits, 2);
        if ((c8 & 3) == 0) s_codes[tok * kWords + (c8 >> 2)] = bits;
      } else {
        bits <<= 16 - 16 * (c8 & 1);
        bits |= __shfl_xor(bits, 1);
        if ((c8 & 1) == 0) s_codes[tok * kWords + (c8 >> 1)] = bits;
      }
    }
    }
  } else {
    // ---- 1. per-token extrema over the lanes of a channel group
    constexpr int kLanesPerGroup = GROUP / 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const v8h xi = x[i];
      const v4h qa = __builtin_shufflevector(xi, xi, 0, 1, 2, 3);
      const v4h qb = __builtin_shufflevector(xi, xi, 4, 5, 6, 7);
      const v4h lo4 = __builtin_elementwise_min(qa, qb), hi4 = __builtin_elementwise_max(qa, qb);
      const v2h lo = __builtin_elementwise_min(__builtin_shufflevector(lo4, lo4, 0, 1),
                                               __builtin_shufflevector(lo4, lo4, 2, 3));
      const v2h hi = __builtin_elementwise_max(__builtin_shufflevector(hi4, hi4, 0, 1),
                                               __builtin_shufflevector(hi4, hi4, 2, 3));
      v2h st = {(_Float16)fminf((float)lo[0], (float)lo[1]),
                (_Float16)(-fmaxf((float)hi[0], (float)hi[1]))};                    // {min, -max}
#pragma unroll
      for (int o = 1; o < kLanesPerGroup; o <<= 1) {
        const uint32_t other = __shfl_xor(__builtin_bit_cast(uint32_t, st), o);
        st = __builtin_elementwise_min(st, __builtin_bit_cast(v2h, other));
      }
      if ((c8 % kLanesPerGroup) == 0) {
        const int tok = 32 * wave + 4 * i + ts;
        s_stat[tok][c8 / kLanesPerGroup][0] = st[0];
        s_stat[tok][c8 / kLanesPerGroup][1] = -st[1];
      }
    }
    __syncthreads();
    // ---- 2. one thread per (token, channel group)
    for (int item = tid; item < kTile * NG; item += kThreads) {
      const int tok = item / NG, g = item % NG;
      const uint16_t mbits = canonical_zero(__builtin_bit_cast(uint16_t, s_stat[tok][g][0]));
      const double alpha = h_to_double(mbits);
      const double D = ((double)(float)s_stat[tok][g][1] - alpha) + 0.0;
      const size_t meta = (tok0 + tok) * NG + g;
      a.scale[meta] = (float)(D / (double)L);
      a.minv[meta] = mbits;
      if constexpr (kWide) {
        s_alpha[tok * 4 + g] = __builtin_bit_cast(_Float16, mbits);
        s_rinv[tok * 4 + g] = D > 0.0 ? (double)L / D : 0.0;
      } else {
#pragma unroll
        for (int k = 1; k <= L; ++k)
          s_thr[(tok * 4 + g) * 4 + (k - 1)] = __builtin_bit_cast(_Float16, threshold_bits(alpha, D, k, L));
      }
    }
    __syncthreads();
    // ---- 3. codes
    const int g = c8 / kLanesPerGroup;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int tok = 32 * wave + 4 * i + ts;
      if constexpr (kWide) {
        const float a32 = (float)s_alpha[tok * 4 + g];
        const double a1 = (double)a32, r1 = s_rinv[tok * 4 + g];
        const float r32 = (float)r1;
        const double al[8] = {a1, a1, a1, a1, a1, a1, a1, a1}, ri[8] = {r1, r1, r1, r1, r1, r1, r1, r1};
        const float al32[8] = {a32, a32, a32, a32, a32, a32, a32, a32};
        const float ri32[8] = {r32, r32, r32, r32, r32, r32, r32, r32};
        uint32_t w0, w1;
        octet_words<BITS>(x[i], al, ri, al32, ri32, w0, w1);
        if constexpr (BITS == 4) {
          s_codes[tok * kWords + c8] = w0;
        } else {
          s_codes[tok * kWords + 2 * c8] = w0;
          s_codes[tok * kWords + 2 * c8 + 1] = w1;
        }
        continue;
      }
      v8h thr[L];
#pragma unroll
      for (int k = 0; k < L; ++k) {
        const _Float16 t = s_thr[(tok * 4 + g) * 4 + k];
        thr[k] = (v8h){t, t, t, t, t, t, t, t};
      }
      uint32_t bits = octet_codes<BITS>(x[i], thr);
      if constexpr (BITS == 1) {
        bits <<= 24 - 8 * (c8 & 3);
        bits |= __shfl_xor(bits, 1);
        bits |= __shfl_xor(bits, 2);
        if ((c8 & 3) == 0) s_codes[tok * kWords + (c8 >> 2)] = bits;
      } else {
        bits <<= 16 - 16 * (c8 & 1);
        bits |= __shfl_xor(bits, 1);
        if ((c8 & 1) == 0) s_codes[tok * kWords + (c8 >> 1)] = bits;
      }
    }
  }
  __syncthreads();
  // ---- the tile's words are contiguous in memory: 16 bytes per thread
  v4u* dst = reinterpret_cast<v4u*>(a.codes + tok0 * kWords);
  for (int i = tid; i < kTile * kWords / 4; i += kThreads)
    dst[i] = *reinterpret_cast<const v4u*>(&s_codes[i * 4]);
}

template <int AXIS, int BITS>
hipError_t launch_group(int group, const QArgs& a, unsigned blocks, hipStream_t stream) {
  switch (group) {
    case 32: quantize_tile_kernel<AXIS, BITS, 32><<<dim3(blocks), dim3(kThreads), 0, stream>>>(a); break;
    case 64: quantize_tile_kernel<AXIS, BITS, 64><<<dim3(blocks), dim3(kThreads), 0, stream>>>(a); break;
    case 128: quantize_tile_kernel<AXIS, BITS, 128><<<dim3(blocks), dim3(kThreads), 0, stream>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// whole-sequence statistics: extrema pass, all tiles but the last of every row, the last tiles
template <int BITS>
hipError_t launch_whole(QArgs a, unsigned rows, hipStream_t stream) {
  row_extrema_kernel<BITS><<<dim3(rows * kSplits), dim3(kThreads), 0, stream>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  a.tile_first = 0;
  a.tiles_launch = a.tiles_row - 1;
  {
    const unsigned long long blocks = (unsigned long long)rows * (unsigned)a.tiles_launch;
    a.launch_magic = a.tiles_launch > 1 && blocks * (unsigned)a.tiles_launch < (1ull << 32)
                         ? (unsigned)((1ull << 32) / (unsigned)a.tiles_launch + 1) : 0u;
  }
  quantize_tile_kernel<CQ_AXIS_CHANNEL, BITS, 0>
      <<<dim3(rows * (unsigned)a.tiles_launch), dim3(kThreads), 0, stream>>>(a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  a.tile_first = a.tiles_row - 1;
  a.tiles_launch = 1;
  a.launch_magic = 0;
  quantize_tile_kernel<CQ_AXIS_CHANNEL, BITS, 0><<<dim3(rows), dim3(kThreads), 0, stream>>>(a);
  return hipGetLastError();
}

}  // namespace

bool quantize_tuned_supported(int n_vis, int d, int bits, int axis, int group) {
  if (d != kD || (bits != 1 && bits != 2 && bits != 4 && bits != 8)) return false;
  if (axis != CQ_AXIS_CHANNEL && axis != CQ_AXIS_TOKEN) return false;
  if (n_vis <= 0 || n_vis % kTile != 0) return false;
  if (axis == CQ_AXIS_CHANNEL && group == n_vis && n_vis > kTile) return true;   // whole sequence
  return group == 32 || group == 64 || group == 128;
}

hipError_t launch_quantize_tuned(const void* x_f16, const cq_qtensor_t& out, int rows, int n_vis,
                                 int bits, int axis, int group, hipStream_t stream) {
  const size_t blocks = (size_t)rows * (size_t)(n_vis / kTile);
  if (blocks > 0x7fffffffu) return hipErrorInvalidConfiguration;
  const QArgs a{static_cast<const __half*>(x_f16), out.codes, out.scale, out.min, n_vis / kTile, 0, 0};
  const unsigned nb = (unsigned)blocks;
  if (axis == CQ_AXIS_CHANNEL && group == n_vis && n_vis > kTile) {
    switch (bits) {
      case 1: return launch_whole<1>(a, (unsigned)rows, stream);
      case 2: return launch_whole<2>(a, (unsigned)rows, stream);
      case 4: return launch_whole<4>(a, (unsigned)rows, stream);
      case 8: return launch_whole<8>(a, (unsigned)rows, stream);
    }
    return hipErrorInvalidValue;
  }
  if (axis == CQ_AXIS_CHANNEL) {
    switch (bits) {
      case 1: return launch_group<CQ_AXIS_CHANNEL, 1>(group, a, nb, stream);
      case 2: return launch_group<CQ_AXIS_CHANNEL, 2>(group, a, nb, stream);
      case 4: return launch_group<CQ_AXIS_CHANNEL, 4>(group, a, nb, stream);
      case 8: return launch_group<CQ_AXIS_CHANNEL, 8>(group, a, nb, stream);
    }
  } else {
    switch (bits) {
      case 1: return launch_group<CQ_AXIS_TOKEN, 1>(group, a, nb, stream);
      case 2: return launch_group<CQ_AXIS_TOKEN, 2>(group, a, nb, stream);
      case 4: return launch_group<CQ_AXIS_TOKEN, 4>(group, a, nb, stream);
      case 8: return launch_group<CQ_AXIS_TOKEN, 8>(group, a, nb, stream);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace cq
