// Streaming decode attention for rows that one workgroup cannot own (gfx950): head_dim 128, 1- or
// 2-bit codes, channel-wise keys in groups of 128 tokens, token-wise values, up to 8 query heads
// per KV head.
//
// The dynamic calibration of Sec. 3.2 needs gamma, delta = the extrema of ALL visual logits of a
// query row before any weight can be formed, so a row that is spread over several workgroups
// takes two passes.  Here the passes are two kernels that meet in memory, and neither keeps
// logits on chip, so both stream with small workgroups, several of them resident per CU:
//
//   logits pass   (row, chunk of key groups) per workgroup of 4 waves.  Post-scaled logits of
//                 Sec. 3.1 from the packed keys on the int8 matrix cores (the contraction of
//                 decode_fused.hip: AND-mask operands, query as four base-256 digits), for ALL
//                 query heads of the KV head at once: a second operand set for heads 4..7 reuses
//                 the expanded code operands, which is most of the vector work.  Raw logits go to
//                 the workspace in 16 bits (below), chunk extrema as [B*Hq][chunks][2].
//   values pass   (row, chunk of key groups) per workgroup of 4 waves on the packed values, (row,
//                 chunk of the fp16 tail) per workgroup of 4 text waves.  Every visual wave folds
//                 the row's extrema, forms g (Sec. 3.2) and the reference point; the visual waves
//                 read logits and packed values, exponentiate and accumulate the weighted value
//                 sum on the int8 matrix cores (weights p_j * scale_j as base-256 digits, both head
//                 sets against the same expanded value operands).  The text waves take the chunk's
//                 share of the fp16 tail from logits to values on the fp16 matrix cores, each
//                 wave on token shares of its own with its own reference point, so no barrier
//                 separates anything before the epilogue, which merges the waves' partial sums
//                 into one (m, l, acc[128]) per (head, chunk).
//   combine       the shared kernel of decode_generic.hip (online-softmax merge over chunks).
//
// Against recomputing the logits in the second pass (what decode_fused.hip does for split rows)
// this trades a second read of the packed keys (16b + 6 bytes per token) and all of its
// arithmetic for 2g bytes of logits per token written and read once.
//
// Logits in 16 bits.  What a weight needs from its logit is absolute accuracy in proportion to the
// weight itself, and the weights that count belong to the largest logits.  So a logit s of key
// group G and head h is kept as its distance e = ref - s >= 0 to the group's own maximum
// ref[h][G] (fp32, one per group and head), rounded to fp16: a token at distance e < 1 of its
// group's maximum is off by at most 2^-12, one at distance 4..8 by 2^-9 with a weight below
// e^-4 of the maximum's, so the error in units of the largest weight stays below 2e-4 however
// wide the range of the logits is (a uniform 16-bit grid over a range of 100, which heavy-tailed
// keys reach, would be off by 8e-4 everywhere), and a group far below the row's maximum does not
// matter at all.  When the calibration line is known on the host to FALL (CQ_CALIB_FIXED with
// delta - gamma + tau1 - tau2 < 0, applied literally), the smallest logits get the largest weights
// and ref is the group's minimum, e = s - ref.  With CQ_CALIB_DYNAMIC a falling line needs a range
// below tau2 - tau1, where every distance is small.  The 128 tokens of a group are stored in the
// order (tile pair, token of the tile, tile of the pair), so that a lane of the logits pass
// writes two logits with one 4-byte store.
#include <hip/hip_fp16.h>

#include <atomic>
#include <cfloat>
#include <type_traits>

#include "cq_internal.h"
#include "decode_device.h"

namespace cq {
namespace {

constexpr int kAWaves = 4;                       // logits pass: waves per workgroup
constexpr int kAThreads = kAWaves * 64;
// values pass: a workgroup is four waves that all stream the packed values of a chunk, or four
// waves that all stream a chunk of the fp16 tail (one wave per SIMD and workgroup, so that three
// workgroups fit a CU at 168 registers per lane whatever mix of the two arrives)
constexpr int kBWaves = 4;
constexpr int kBVisWaves = kBWaves, kBTextWaves = kBWaves;
constexpr int kBThreads = kBWaves * 64;
constexpr int kRing = 2;                         // key groups / value tiles in flight per wave
constexpr int kRingTK = 2, kRingTV = 4;          // text key tiles / text value steps in flight
typedef _Float16 v2h16 __attribute__((ext_vector_type(2)));

struct StreamArgs {
  const __half* q;
  const uint32_t* k_codes; const float* k_scale; const uint16_t* k_min;
  const uint32_t* v_codes; const float* v_scale; const uint16_t* v_min;
  const __half* k_text; const __half* v_text;
  int g, n_vis, n_text, n_text_cap;
  const int32_t* n_text_dev;     // NULL, or the tail length in device memory (n_text is its bound)
  // logits pass: ca chunks per row, in units of key groups (128 tokens)
  int ca, ca_base, ca_rem; unsigned ca_magic;
  // values pass: cb chunks of key groups per row, ct chunks of 64-token text blocks per row; the
  // first n_text_wg workgroups of the launch take the text chunks
  int cb, cb_base, cb_rem; unsigned cb_magic;
  int ct, tb_base, tb_rem, n_text_wg; unsigned ct_magic;
  int tstride;                   // floats between the text-logit rows of two heads in LDS
  float* ws_minmax;              // [B*Hq][ca][2]  extrema of each chunk's visual logits
  float* ws_lref;                // [B*Hq][n_vis / 128]  reference logit of each key group
  uint16_t* ws_logits;           // [B*Hq][n_vis]  fp16 distances of the raw visual logits to it
  int falling;                   // the reference is the group's minimum (falling calibration line)
  int ref_stride;                // values pass: key groups of the largest chunk (sizes the LDS table)
  float* ws_partial;             // [B*Hq][cb][d + 2]  (m, l, acc) for the combine
  int calib_mode; float tau1, tau2, gamma, delta, softmax_scale;
};

extern __shared__ __align__(16) uint8_t smem[];

// Maximum / minimum over each row of 16 lanes, every lane gets the result.  Written out because
// the compiler puts a canonicalising v_max in front of every fmaxf whose operand went through a
// DPP move and then cannot fold the move into the maximum: three instructions per step instead of
// one.  The inputs here are finite results of arithmetic.  (Two idle states separate a vector
// write from a DPP read of the same register.)
#define CQ_ROW_REDUCE(OP)                                                                        \
  float r;                                                                                       \
  asm volatile("s_nop 1\n\t" OP " %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t" \
               "s_nop 1\n\t" OP " %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t" \
               "s_nop 1\n\t" OP " %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"    \
               "s_nop 1\n\t" OP " %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf"               \
               : "=&v"(r)                                                                        \
               : "v"(v));                                                                        \
  return r;
__device__ __forceinline__ float row_max_finite(float v) { CQ_ROW_REDUCE("v_max_f32_dpp") }
__device__ __forceinline__ float row_min_finite(float v) { CQ_ROW_REDUCE("v_min_f32_dpp") }
#undef CQ_ROW_REDUCE

// ===================================================================================== logits pass
// BITS = code width (1 or 2); NS = sets of 4 query heads (1 or 2: g <= 4 or g <= 8).
// (one head set leaves room for four waves per SIMD, two need the registers of three)
template <int BITS, int NS>
__global__ void __launch_bounds__(kAThreads) __attribute__((amdgpu_waves_per_eu(NS == 1 ? 4 : 3, NS == 1 ? 4 : 3)))
stream_logits_kernel(const StreamArgs a) {
  constexpr int TILES = 8;                       // 16-token tiles per key group
  constexpr int kV = 8 / BITS, kCW = 32 / BITS;  // variants per byte, codes per word
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n16 = lane & 15, kb = lane >> 4;
  const int piece = blockIdx.x;
  const int row = a.ca_magic ? (int)__umulhi((unsigned)piece, a.ca_magic) : piece;
  const int chunk = piece - row * a.ca;
  const int ga = chunk_first(a.ca_base, a.ca_rem, chunk), gb = chunk_first(a.ca_base, a.ca_rem, chunk + 1);
  const int n_groups = gb - ga;
  const size_t head0 = (size_t)row * a.g;

  // ---- LDS: the query (fp32), one operand staging buffer per (wave, head set), reduction slots
  float* qf = reinterpret_cast<float*>(smem);                          // [NS * 4][128]
  uint8_t* stage = smem + NS * kHeads * kD * 4 + (size_t)wave * (NS * 2048);
  float* red_q = reinterpret_cast<float*>(smem + NS * kHeads * kD * 4 + kAWaves * NS * 2048);   // [2 NS][waves]
  float* red_m = red_q + 2 * NS * kAWaves;                             // [waves][NS * 4][2]

  // ---- query to LDS and max |q| per head set (bounds the fixed-point operand of a key group)
#pragma unroll
  for (int i = 0; i < 2 * NS; ++i) {             // pass i: heads 2i (waves 0, 1) and 2i + 1 (waves 2, 3)
    const int e = tid + kAThreads * i, h = e >> 7;
    const float qv = h < a.g ? __half2float(a.q[(head0 + h) * kD + (e & 127)]) : 0.f;
    qf[e] = qv;
    const float m = wave_max_nonneg(fabsf(qv));
    if (lane == 0) red_q[i * kAWaves + wave] = m;
  }
  __syncthreads();
  float qmax[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    float m = 0.f;
#pragma unroll
    for (int j = 0; j < 2 * kAWaves; ++j) m = fmaxf(m, red_q[2 * s * kAWaves + j]);
    qmax[s] = m * a.softmax_scale;
  }

  // Lane roles (as in the fused kernel): the writer of the query operand handles the two adjacent
  // channels wc0, wc1 (their scales and minima arrive with one coalesced load each); matrix lane
  // (n16, kb) holds token n16 of a tile and word(s) kb of it; result lane (n16, kb) holds token
  // n16 for head kb of each set.
  const int wc0 = 32 * kb + 2 * n16, wc1 = wc0 + 1;
  auto row_of = [&](int c, int& variant) {       // operand row inside the kb block, and its variant
    const int cl = c & 31, e = cl / kCW, t = kCW - 1 - cl % kCW;
    const int y = t / kV, v = t % kV, pair = e * kV + v;
    variant = v;
    return pair * 4 + y;
  };
  int wvar0, wvar1;
  const int wr0 = row_of(wc0, wvar0), wr1 = row_of(wc1, wvar1);
  const float inv_w0 = 1.f / variant_weight<BITS>(wvar0), inv_w1 = 1.f / variant_weight<BITS>(wvar1);
  const int x_wr0 = kb * 512 + wr0 * 16, x_wr1 = kb * 512 + wr1 * 16;
  const int x_rd = kb * 512 + (n16 >> 1) * 16 + (n16 & 1) * 8;
  const size_t tok0 = (size_t)row * a.n_vis + (size_t)ga * 128;        // first token of the chunk
  const uint32_t* kq_lane = a.k_codes + tok0 * 4 + (size_t)(16 * kb + n16) * 4;              // b = 1
  const uint32_t* kc_lane = a.k_codes + tok0 * (4 * BITS) + n16 * (4 * BITS) + kb * BITS;    // b = 2
  const float* ks_row = a.k_scale + ((size_t)row * (a.n_vis >> 7) + ga) * kD;
  const uint16_t* km_row = a.k_min + ((size_t)row * (a.n_vis >> 7) + ga) * kD;
  // Where this lane's results go: head 4s + kb, token n16 of each tile.  Stores go through buffer
  // descriptors that cover the row's g heads: the lanes of heads that do not exist (g not a
  // multiple of 4) compute along on a zero query and their stores fall outside and are dropped,
  // so nothing branches.  Token (tile i, n16) of a group sits at ((i % 4) * 16 + n16) * 2 + i / 4:
  // a 4-byte word holds the same token of the group's two 64-token halves, which is what a lane
  // of the values pass wants.
  const int n_grow = a.n_vis >> 7;               // key groups per row
  const __amdgpu_buffer_rsrc_t lbuf =
      stream_buffer(a.ws_logits + head0 * (size_t)a.n_vis, (unsigned)((size_t)a.g * a.n_vis * 2));
  const __amdgpu_buffer_rsrc_t rbuf =
      stream_buffer(a.ws_lref + head0 * (size_t)n_grow, (unsigned)((size_t)a.g * n_grow * 4));
  int l_off[NS], r_off[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    l_off[s] = ((4 * s + kb) * a.n_vis + ga * 128 + 2 * n16) * 2;      // word n16 of a tile pair
    r_off[s] = n16 == 0 ? ((4 * s + kb) * n_grow + ga) * 4 : 0x7ffffff0;    // one lane per head writes
  }

  constexpr bool kQuadKeys = BITS == 1;          // 16-byte loads over four tiles, see decode_fused.hip
  uint32_t w[kQuadKeys ? 1 : kRing][TILES][BITS];
  v4i wq[kQuadKeys ? kRing : 1][2];
  v2f s01[kRing];
  uint32_t m01[kRing];
  auto load_group = [&](int slot, int t) {
    const int tc = min(t, n_groups - 1);         // clamped, never a branch around a load
    if constexpr (kQuadKeys) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
        wq[slot][j] = stream_load<true>(reinterpret_cast<const v4i*>(kq_lane + ((size_t)tc * TILES + 4 * j) * 64));
    } else {
#pragma unroll
      for (int i = 0; i < TILES; ++i) {
        const v2i t2 = stream_load<true>(reinterpret_cast<const v2i*>(kc_lane + ((size_t)tc * TILES + i) * (64 * BITS)));
        w[slot][i][0] = (uint32_t)t2[0];
        w[slot][i][BITS - 1] = (uint32_t)t2[1];
      }
    }
    s01[slot] = stream_load<true>(reinterpret_cast<const v2f*>(ks_row + (size_t)tc * kD + wc0));
    m01[slot] = stream_load<true>(reinterpret_cast<const uint32_t*>(km_row + (size_t)tc * kD + wc0));
  };

  float qv0[NS][kHeads], qv1[NS][kHeads];
  float mn[NS], mx[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) { mn[s] = FLT_MAX; mx[s] = -FLT_MAX; }

  auto do_group = [&](int slot, int t) {
    // query operands of the group, one set of 16 matrix rows (4 heads x 4 digits) per head set
    const float s0 = s01[slot][0], s1 = s01[slot][1];
    const float smax = wave_max_nonneg(fmaxf(s0, s1));
    v4i A0[NS], A1[NS];
    float bias_h[NS], inv_f[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int F = fixed_point_shift(qmax[s] * smax);
      const float s0f = ldexpf(s0, F), s1f = ldexpf(s1, F);
      v4i x0, x1;
#pragma unroll
      for (int h = 0; h < kHeads; ++h) {
        x0[h] = product_digits(qv0[s][h], s0f);
        x1[h] = product_digits(qv1[s][h], s1f);
      }
      inv_f[s] = ldexpf(1.f, -F);
      uint8_t* xb = stage + s * 2048;
      __builtin_amdgcn_wave_barrier();
      *reinterpret_cast<v4i*>(xb + x_wr0) = x0;
      *reinterpret_cast<v4i*>(xb + x_wr1) = x1;
      lds_publish();
      const uint8_t* xr = xb + x_rd;
      const v2i r00 = lds_read_tr8(xr), r01 = lds_read_tr8(xr + 128);
      const v2i r10 = lds_read_tr8(xr + 256), r11 = lds_read_tr8(xr + 384);
      A0[s] = (v4i){r00[0], r00[1], r01[0], r01[1]};
      A1[s] = (v4i){r10[0], r10[1], r11[0], r11[1]};
      bias_h[s] = group_bias(qv0[s], qv1[s], (uint16_t)(m01[slot] & 0xffffu), (uint16_t)(m01[slot] >> 16),
                             0.f, 0.f, inv_w0, inv_w1, lane);
    }
    __builtin_amdgcn_wave_barrier();
    uint32_t wt[TILES];                          // one-bit keys: the lane's word of every tile
    if constexpr (kQuadKeys) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const v4i raw = wq[slot][j];
        v2u lo = __builtin_amdgcn_permlane32_swap((unsigned)raw[0], (unsigned)raw[2], false, false);
        v2u hi = __builtin_amdgcn_permlane32_swap((unsigned)raw[1], (unsigned)raw[3], false, false);
        const v2u t01 = __builtin_amdgcn_permlane16_swap(lo[0], hi[0], false, false);
        const v2u t23 = __builtin_amdgcn_permlane16_swap(lo[1], hi[1], false, false);
        wt[4 * j + 0] = t01[0];
        wt[4 * j + 1] = t01[1];
        wt[4 * j + 2] = t23[0];
        wt[4 * j + 3] = t23[1];
      }
    }
    auto expand = [&](int tile, v4i& B0, v4i& B1) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        if constexpr (kQuadKeys) {
          B0[v] = operand_variant<BITS>(wt[tile], v);
          B1[v] = operand_variant<BITS>(wt[tile], 4 + v);
        } else {
          B0[v] = operand_variant<BITS>(w[slot][tile][v / kV], v % kV);
          B1[v] = operand_variant<BITS>(w[slot][tile][(4 + v) / kV], (4 + v) % kV);
        }
      }
    };
    // The group's logits of this lane stay in units of 2^-F until the group is done: u = the
    // integer the digit accumulators spell, logit = u * 2^-F + bias.  Scale and bias are the same
    // for every token of the group and head and the scale is positive, so extrema and distances
    // are taken on u and converted once.
    float sv[NS][TILES], gmn[NS], gmx[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) { gmn[s] = FLT_MAX; gmx[s] = -FLT_MAX; }
    auto finish_tile = [&](int s, int tile, const v4i& c) {
      const int lo = c[0] + (c[1] << 8), hi = c[2] + (c[3] << 8);
      const float u = fmaf((float)hi, 65536.f, (float)lo);
      sv[s][tile] = u;
      gmn[s] = fminf(gmn[s], u);
      gmx[s] = fmaxf(gmx[s], u);
    };
#pragma unroll
    for (int tile = 0; tile < TILES; tile += 2) {
      v4i Ba0, Ba1, Bb0, Bb1;
      expand(tile, Ba0, Ba1);
      expand(tile + 1, Bb0, Bb1);
      __builtin_amdgcn_sched_barrier(0);
      v4i ca[NS], cb[NS];
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const v4i z = {0, 0, 0, 0};
        ca[s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A0[s], Ba0, z, 0, 0, 0);
        cb[s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A0[s], Bb0, z, 0, 0, 0);
      }
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        ca[s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A1[s], Ba1, ca[s], 0, 0, 0);
        cb[s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A1[s], Bb1, cb[s], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        finish_tile(s, tile, ca[s]);
        finish_tile(s, tile + 1, cb[s]);
      }
    }
    // the group's reference logit per head (its maximum, or its minimum under a falling
    // calibration line) and the fp16 distances to it, two tokens per store
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      mn[s] = fminf(mn[s], fmaf(gmn[s], inv_f[s], bias_h[s]));
      mx[s] = fmaxf(mx[s], fmaf(gmx[s], inv_f[s], bias_h[s]));
      const float ref_u = a.falling ? row_min_finite(gmn[s]) : row_max_finite(gmx[s]);
      const float ref = fmaf(ref_u, inv_f[s], bias_h[s]);
      __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, ref), rbuf, r_off[s], t * 4, 0);
      // distance e = |ref_u - u| 2^-F = k u - k ref_u with k = -+2^-F
      const float k = a.falling ? inv_f[s] : -inv_f[s];
      const float c0 = -k * ref_u;
#pragma unroll
      for (int pr = 0; pr < TILES / 2; ++pr) {
        const v2h16 e = {(_Float16)fmaf(sv[s][pr], k, c0), (_Float16)fmaf(sv[s][pr + 4], k, c0)};
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, e), lbuf, l_off[s],
                                              (t * 128 + pr * 32) * 2, 0);
      }
    }
  };

#pragma unroll
  for (int d = 0; d < kRing; ++d) load_group(d, wave + d * kAWaves);
  pin_order();
  // the lane's slice of the staged query, read while the first key groups are on their way
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int h = 0; h < kHeads; ++h) {
      qv0[s][h] = qf[(4 * s + h) * kD + wc0] * (a.softmax_scale * variant_weight<BITS>(wvar0));
      qv1[s][h] = qf[(4 * s + h) * kD + wc1] * (a.softmax_scale * variant_weight<BITS>(wvar1));
    }
  int t = wave;
  for (; t + (kRing - 1) * kAWaves < n_groups; t += kRing * kAWaves) {
#pragma unroll
    for (int d = 0; d < kRing; ++d) {            // no branch around the ring's loads
      const int tt = t + d * kAWaves;
      do_group(d, tt);
      pin_order();
      load_group(d, tt + kRing * kAWaves);
      pin_order();
    }
  }
#pragma unroll
  for (int d = 0; d < kRing; ++d)                // the wave's last groups, already loaded
    if (t + d * kAWaves < n_groups) do_group(d, t + d * kAWaves);

  // ---- extrema of the chunk: 16 token lanes per head on the DPP network, then over the waves
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const float lo = row_min(mn[s]), hi = row_max(mx[s]);
    if (n16 == 0) {
      red_m[((wave * NS + s) * kHeads + kb) * 2 + 0] = lo;
      red_m[((wave * NS + s) * kHeads + kb) * 2 + 1] = hi;
    }
  }
  __syncthreads();
  if (tid < NS * kHeads && tid < a.g) {          // tid = head 4s + kb
    float lo = FLT_MAX, hi = -FLT_MAX;
    for (int wv = 0; wv < kAWaves; ++wv) {
      lo = fminf(lo, red_m[(wv * NS * kHeads + tid) * 2 + 0]);
      hi = fmaxf(hi, red_m[(wv * NS * kHeads + tid) * 2 + 1]);
    }
    float* mm = a.ws_minmax + ((head0 + tid) * a.ca + chunk) * 2;
    mm[0] = lo;
    mm[1] = hi;
  }
}

// ===================================================================================== values pass
// HL = heads that exist in the last head set (g - 4 (NS - 1)): the weights of head slots without a
// head are not computed at all.  ONE = one register slot for the packed values in flight instead
// of two (with two head sets, where two slots spill).
template <int BITS, int NS, int HL, bool ONE>
__global__ void __launch_bounds__(kBThreads) __attribute__((amdgpu_waves_per_eu(NS == 1 ? 4 : 3, NS == 1 ? 4 : 3)))
stream_values_kernel(const StreamArgs a) {
  static_assert(HL >= 1 && HL <= kHeads, "see above");
  constexpr int NH = NS * kHeads;                // head slots of the workgroup
  constexpr int kSlots = kHeads * (NS - 1) + HL;           // head slots that hold a head
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n16 = lane & 15, kb = lane >> 4;
  // workgroup = (row, chunk of the fp16 tail) for the first n_text_wg of them, then (row, chunk of
  // key groups): the text chunks, which depend on nothing, start first
  const bool text_wg = (int)blockIdx.x < a.n_text_wg;
  const int piece = text_wg ? (int)blockIdx.x : (int)blockIdx.x - a.n_text_wg;
  const unsigned magic = text_wg ? a.ct_magic : a.cb_magic;
  const int per_row = text_wg ? a.ct : a.cb;
  const int row = magic ? (int)__umulhi((unsigned)piece, magic) : piece;
  const int chunk = piece - row * per_row;
  const size_t head0 = (size_t)row * a.g;
  const int n_slots = a.cb + a.ct;               // partials per head: key-group chunks, then text chunks
  const int slot = text_wg ? a.cb + chunk : chunk;
  // a visual workgroup: the chunk's key groups (128 tokens: two 64-token value tiles)
  const int ga = text_wg ? 0 : chunk_first(a.cb_base, a.cb_rem, chunk);
  const int n_gchunk = text_wg ? 0 : chunk_first(a.cb_base, a.cb_rem, chunk + 1) - ga;
  // a text workgroup: the chunk's 64-token blocks of the tail
  const int n_text = a.n_text_dev ? min(max(*a.n_text_dev, 0), a.n_text) : a.n_text;
  const int ba = chunk_first(a.tb_base, a.tb_rem, chunk), bb = chunk_first(a.tb_base, a.tb_rem, chunk + 1);
  const int txt0 = ba * 64;
  const int ntx = text_wg ? max(0, min(n_text, bb * 64) - txt0) : 0;
  const bool vis_wave = !text_wg;
  const int tw = wave;

  // ---- LDS: staging of the visual waves (weights as digits per head set, code bytes), the text
  // logits, every wave's partial sums for the epilogue, the chunk's table of group constants
  constexpr int kStage = NS * 1024 + 2048;
  uint8_t* stage = smem + (size_t)wave * kStage;
  float* tlog = reinterpret_cast<float*>(smem + kBVisWaves * kStage);          // [NH][tstride]
  uint8_t* tbytes = reinterpret_cast<uint8_t*>(tlog);
  float* partial = tlog + (size_t)NH * a.tstride + (size_t)wave * NH * kD;    // [waves][NH][128]
  float* mla = tlog + (size_t)NH * a.tstride + (size_t)kBWaves * NH * kD;     // [waves][NH][3]: m, l, additive
  float* ref_tab = mla + kBWaves * NH * 3;                                     // [groups of the chunk][NH]
  const int n_grow = a.n_vis >> 7;

  // ---- calibration line and reference point of the visual logits, per head (Sec. 3.2).  Every
  // wave folds the row's chunk extrema of the logits pass itself: lane 16j + c takes chunks c,
  // c + 16, ... of head 4s + j.
  float a2[NH], c2v[NH];
  const bool vis_work = vis_wave && wave < n_gchunk;      // the wave owns at least one key group
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    if (text_wg) {                               // nothing of this concerns the tail
#pragma unroll
      for (int j = 0; j < kHeads; ++j) { a2[4 * s + j] = 0.f; c2v[4 * s + j] = 0.f; }
      continue;
    }
    const int h = min(4 * s + kb, a.g - 1);
    const float* mm = a.ws_minmax + (head0 + h) * (size_t)a.ca * 2;
    float lo_l = FLT_MAX, hi_l = -FLT_MAX;
    for (int c = n16; c < a.ca; c += 16) {
      lo_l = fminf(lo_l, mm[2 * c]);
      hi_l = fmaxf(hi_l, mm[2 * c + 1]);
    }
    lo_l = row_min(lo_l);
    hi_l = row_max(hi_l);
#pragma unroll
    for (int j = 0; j < kHeads; ++j) {
      const float lo = lane_value(lo_l, 16 * j), hi = lane_value(hi_l, 16 * j);
      float slope = 1.f, gam = 0.f, shift = 0.f;       // s' = slope * (s - gam) + shift
      if (a.calib_mode != CQ_CALIB_NONE) {
        const float glo = a.calib_mode == CQ_CALIB_DYNAMIC ? lo : a.gamma;
        const float ghi = a.calib_mode == CQ_CALIB_DYNAMIC ? hi : a.delta;
        const float width = ghi - glo;
        slope = width == 0.f ? 1.f : (width + a.tau1 - a.tau2) / width;
        gam = glo;
        shift = glo - a.tau1;
      }
      // the map is monotone: an end point of the row's range is its maximum, every weight <= 1.
      // All chunks of a row share this reference point.
      const float M = fmaxf(slope * (lo - gam) + shift, slope * (hi - gam) + shift);
      const bool exists = 4 * s + j < a.g;
      if (vis_wave && lane == 0)
        mla[(wave * NH + 4 * s + j) * 3] = vis_work ? M : -FLT_MAX;
      // exponent of a weight in base 2: a2 * s + c2v
      a2[4 * s + j] = exists ? slope * kLog2e : 0.f;
      c2v[4 * s + j] = exists ? (shift - slope * gam - M) * kLog2e : -200.f;   // no head: weight 0
    }
  }

  // The logits pass keeps a logit as its distance e to the reference logit of its key group:
  // s = ref + dsign e, so the exponent (base 2) of a weight is na2 e + (a2 ref + c2v).  The second
  // term is the same for all tokens of a group: one table per head for the chunk's groups.
  const float dsign = a.falling ? 1.f : -1.f;
  for (int e = tid; e < NH * n_gchunk; e += kBThreads) {
    const int h = e / n_gchunk, gi = e - h * n_gchunk;
    float a2h = 0.f, c2h = 0.f;
#pragma unroll
    for (int hh = 0; hh < NH; ++hh)
      if (hh == h) { a2h = a2[hh]; c2h = c2v[hh]; }
    const float ref = a.ws_lref[(head0 + min(h, a.g - 1)) * (size_t)n_grow + ga + gi];
    ref_tab[gi * NH + h] = fmaf(a2h, ref, c2h);
  }
  // a visual wave fills the rows of its own head set only: the rest must read as zeros
  if (vis_wave)
    for (int i = lane; i < NH * kD; i += 64) partial[i] = 0.f;
  __syncthreads();

  float lsum[NH], msum[NH], mref[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) { lsum[h] = 0.f; msum[h] = 0.f; mref[h] = -FLT_MAX; }
  bool wrote = vis_work;       // this wave leaves partial sums in LDS (wave-uniform)

  if (vis_wave) {
    // A visual wave works for all NS head sets at once (both sets against the same expanded value
    // operands).  Pipeline over the wave's key groups (group k of the wave is group
    // wave + kBVisWaves k of the chunk), two 64-token tiles each, tile u = 2k + T, as in the fused
    // kernel:
    //   G(u)  global loads of the tile's codes, scales and minima into a ring of two slots (slot T),
    //         and once per group of the stored logit distances of both tiles (one 4-byte load per
    //         head: the low half is tile 0's token `lane`, the high half tile 1's)
    //   P(u)  weights p = 2^(na2 e + c), their fixed-point digits X(u) and the code bytes to LDS
    //   M(u)  transposing reads of X(u) (per set) and of the codes, 8 x (4 AND + NS MFMA)
    // One step runs M(u), P(u+1) and G(u+3); the distances are asked for two groups ahead.
    constexpr int WH = NH;                       // head slots of the wave
    float na2[WH];                               // wave-uniform: kept in scalar registers
#pragma unroll
    for (int j = 0; j < WH; ++j) {
      float v = a2[j];
      na2[j] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, v * dsign)));
    }
    v4i acc[NS][8];
    float facc[NS][8];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int p = 0; p < 8; ++p) { acc[s][p] = (v4i){0, 0, 0, 0}; facc[s][p] = 0.f; }
    int F_prep = 90, F_acc = 90, F_tile[2] = {90, 90};
    float fit_below = ldexpf(1.f, 29 - 90);      // scales below this fit the shift F_prep
    const int n_my = wave < n_gchunk ? (n_gchunk - wave + kBVisWaves - 1) / kBVisWaves : 0;
    const size_t tok_row = (size_t)row * a.n_vis + (size_t)ga * 128;
    const uint32_t* vc_row = a.v_codes + tok_row * (4 * BITS);
    const float* vs_row = a.v_scale + tok_row;
    const uint16_t* vm_row = a.v_min + tok_row;
    const uint32_t* lg_row[WH];                  // wave-uniform: a row's distances, two tokens per word
#pragma unroll
    for (int j = 0; j < WH; ++j)
      lg_row[j] = reinterpret_cast<const uint32_t*>(a.ws_logits + (head0 + min(j, a.g - 1)) * (size_t)a.n_vis +
                                                    (size_t)ga * 128);
    const int x_rd = kb * 256 + (n16 >> 1) * 16 + (n16 & 1) * 8;
    const int v_rd = (kb * 16 + (n16 >> 1)) * (16 * BITS) + (n16 & 1) * 8;
    uint8_t* xbuf = stage;                        // [NS][1024]: token lane -> 16 bytes (4 heads x 4 digits)
    uint8_t* cbuf = stage + NS * 1024;           // b = 1: two 1 KB buffers alternate; b = 2: one of 2 KB
    // ONE: a single register slot for the tile in flight (loaded one tile ahead instead of two),
    // where two would not fit the registers of three waves per SIMD
    constexpr int kCodeSlots = ONE ? 1 : 2;
    auto sl = [](int T) { return ONE ? 0 : T; };
    v4i cg[kCodeSlots][BITS];
    float vsr[kCodeSlots];
    uint16_t vmr[kCodeSlots];
    // raw fp16 pairs of the current group of the wave and of the next one (converted where used)
    uint32_t lg_cur[WH], lg_next[WH];
    auto group_of = [&](int k) { return wave + kBVisWaves * min(k, n_my - 1); };      // clamped
    auto load_codes = [&](int T, int u) {        // tile u of the wave (T = u % 2) into its slot
      const int j0 = (group_of(u >> 1) * 2 + T) * 64, j = j0 + lane;
#pragma unroll
      for (int e = 0; e < BITS; ++e)
        cg[sl(T)][e] = stream_load<true>(reinterpret_cast<const v4i*>(vc_row + (size_t)j0 * (4 * BITS) + 256 * e + 4 * lane));
      vsr[sl(T)] = stream_load<true>(vs_row + j);
      vmr[sl(T)] = stream_load<true>(vm_row + j);
    };
    auto load_logits = [&](uint32_t (&dst)[WH], int k) {     // group k of the wave
      const int w0 = group_of(k) * 64 + lane;
#pragma unroll
      for (int j = 0; j < kSlots; ++j) dst[j] = stream_load<true>(lg_row[j] + w0);
    };
    auto prep_tile = [&](int T, const uint32_t (&lg)[WH], int k) {   // tile T of the wave's group k
      if (__builtin_amdgcn_ballot_w64(vsr[sl(T)] >= fit_below) != 0) {
        // some token's scale does not fit the running shift (rare after the first tiles)
        F_prep = min(F_prep, fixed_point_shift(wave_max_nonneg(vsr[sl(T)])));
        fit_below = ldexpf(1.f, 29 - F_prep);
      }
      F_tile[T] = F_prep;
      const float vsf = ldexpf(vsr[sl(T)], F_prep);
      float vmf = __half2float(__ushort_as_half(vmr[sl(T)]));
      asm volatile("" : "+v"(vmf));
      const int gi = group_of(k);
      v4i xs[NS];
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        // the group's constants of the set's four heads: one 16-byte LDS read (same address in all lanes)
        const v4f cc = *reinterpret_cast<const v4f*>(ref_tab + gi * NH + 4 * s);
#pragma unroll
        for (int i = 0; i < kHeads; ++i) {
          const int j = 4 * s + i;
          if (j >= kSlots) { xs[s][i] = 0; continue; }     // no such head: zero digits, nothing summed
          const uint32_t pairw = lg[j];
          const float e = __half2float(__ushort_as_half((uint16_t)(T ? pairw >> 16 : pairw & 0xffffu)));
          const float p = __builtin_amdgcn_exp2f(fmaf(e, na2[j], cc[i]));
          lsum[j] += p;
          msum[j] = fmaf(p, vmf, msum[j]);
          xs[s][i] = product_digits(p, vsf);
        }
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int s = 0; s < NS; ++s) *reinterpret_cast<v4i*>(xbuf + s * 1024 + 16 * lane) = xs[s];
#pragma unroll
      for (int e = 0; e < BITS; ++e)
        *reinterpret_cast<v4i*>(cbuf + (BITS == 1 ? T * 1024 : 0) + 1024 * e + 16 * lane) = cg[sl(T)][e];
    };
    // one step: M(tile u = 2k + T) with P(u + 1) and G(u + 3) in its shadow
    auto m_step = [&](int k, int T, bool prep_next) {
      v4i A[NS];
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const uint8_t* xr = xbuf + s * 1024 + x_rd;
        const v2i a_lo = lds_read_tr8(xr), a_hi = lds_read_tr8(xr + 128);
        A[s] = (v4i){a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
      }
      const uint8_t* vr = cbuf + (BITS == 1 ? T * 1024 : 0) + v_rd;
      v4i raw[BITS];
#pragma unroll
      for (int cb = 0; cb < BITS; ++cb) {
        const v2i b_lo = lds_read_tr8(vr + 16 * cb), b_hi = lds_read_tr8(vr + 16 * cb + 128 * BITS);
        raw[cb] = (v4i){b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
      }
      if (T == 0) {
        if (prep_next) prep_tile(1, lg_cur, k);
      } else {
        if (prep_next) prep_tile(0, lg_next, k + 1);
        // the next group becomes the current one; its successor's distances are asked for
#pragma unroll
        for (int j = 0; j < kSlots; ++j) lg_cur[j] = lg_next[j];
      }
      pin_order();
      if constexpr (ONE) load_codes(T, 2 * k + T + 2);        // the slot prep_tile has just emptied
      else load_codes(T ^ 1, 2 * k + T + 3);
      if (T == 1) load_logits(lg_next, k + 2);
      pin_order();
      if (F_tile[T] < F_acc) {                    // wave-uniform, rare: a larger scale lowered the shift
        // bank what was accumulated so far in fp32 (the four digit accumulators of a value
        // cannot be shifted independently)
        const float w_old = ldexpf(1.f, -F_acc);
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
          for (int p = 0; p < 8; ++p) {
            facc[s][p] = fmaf(digits_to_float(acc[s][p]), w_old, facc[s][p]);
            acc[s][p] = (v4i){0, 0, 0, 0};
          }
        F_acc = F_tile[T];
      }
      auto variant_of = [&](int p) {
        v4i B;
#pragma unroll
        for (int v = 0; v < 4; ++v)
          B[v] = operand_variant<BITS>((uint32_t)raw[p / (8 / BITS)][v], p % (8 / BITS));
        return B;
      };
      v4i Bn = variant_of(0);
#pragma unroll
      for (int p = 0; p < 8; ++p) {               // operand p + 1 is formed before product p is issued
        const v4i B = Bn;
        if (p < 7) Bn = variant_of(p + 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < NS; ++s)
          acc[s][p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[s], B, acc[s][p], 0, 0, 0);
      }
      lds_publish();
    };
    if (n_my > 0) {
      load_codes(0, 0);
      if constexpr (!ONE) load_codes(1, 1);
      load_logits(lg_cur, 0);
      load_logits(lg_next, 1);
      pin_order();
      prep_tile(0, lg_cur, 0);
      lds_publish();
      if constexpr (ONE) load_codes(1, 1);
      else load_codes(0, 2);
      pin_order();
      int k = 0;
      for (; k + 1 < n_my; ++k) {                // no branch around a load or a preparation in here
        m_step(k, 0, true);
        m_step(k, 1, true);
      }
      m_step(k, 0, true);                        // the wave's last group
      m_step(k, 1, false);
      // the wave's sums: result lane (column n16 = code byte, head kb of each set), accumulator p
      const float inv_fv = ldexpf(1.f, -F_acc);
#pragma unroll
      for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const float v = fmaf(digits_to_float(acc[s][p]), inv_fv, facc[s][p]);
          constexpr int kV = 8 / BITS;
          const int tbyte = 16 * (p / kV) + n16;
          const int ch = (32 / BITS) * (tbyte >> 2) + code_in_word<BITS>(tbyte & 3, p % kV);
          partial[(4 * s + kb) * kD + ch] = v * variant_weight<BITS>(p % kV);
        }
    }
  } else {
    // ---- text tail of the chunk.  A text wave owns whole shares of SH tokens (share sh = tw,
    // tw + 2, ...): it forms their logits (fp16 matrix cores, 16 heads wide, so all query heads in
    // one product), takes ITS OWN maximum as reference point, and runs the value contraction of
    // the fused kernel on them (4 x 4 x 4 blocks, weights as fp16 pairs hi + lo staged in the
    // share's own logit slots), once per head set on the same loaded values.
    if (ntx > 0) {
      auto text_part = [&](auto share_tag) {
        constexpr int SH = decltype(share_tag)::value;
        constexpr int TPS = SH / 16;             // 16-token logit tiles per share
        const int n_sh = (ntx + SH - 1) / SH;
        const int n_own = n_sh > tw ? (n_sh - tw + kBTextWaves - 1) / kBTextWaves : 0;
        wrote = n_own > 0;
        // -- logits of the wave's own shares
        float tmax[4] = {-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX};     // heads 4 kb + r
        if (n_own > 0) {
          v8h At[4];
#pragma unroll
          for (int s4 = 0; s4 < 4; ++s4) {
            const v8h z = {0, 0, 0, 0, 0, 0, 0, 0};
            At[s4] = n16 < a.g ? *reinterpret_cast<const v8h*>(a.q + (head0 + n16) * kD + 32 * s4 + 8 * kb) : z;
          }
          // a wave-wide load covers one 128-byte line of 8 tokens twice (see the fused kernel):
          // matrix columns n16 and n16 + 8 hold the same token with different channels
          const int tsub = n16 & 7, hsel = n16 >> 3;
          const __amdgpu_buffer_rsrc_t kt_buf =
              stream_buffer(a.k_text + ((size_t)row * a.n_text_cap + txt0) * kD, (unsigned)ntx * kD * 2);
          const int kt_lane = (tsub * kD + 32 * hsel + 8 * kb) * 2;
          const int n_tiles = n_own * TPS;
          auto tile_of = [&](int i) { return (tw + kBTextWaves * (i / TPS)) * TPS + i % TPS; };
          v8h kt[kRingTK][4];
          auto load_tile = [&](int slot, int i) {
            const int tile = tile_of(i);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
              const int tok_bytes = (tile * 16 + 8 * u) * (kD * 2);
              kt[slot][2 * u] = buffer_load_v8h<true>(kt_buf, kt_lane, tok_bytes);
              kt[slot][2 * u + 1] = buffer_load_v8h<true>(kt_buf, kt_lane + 128, tok_bytes);
            }
          };
#pragma unroll
          for (int d = 0; d < kRingTK; ++d) load_tile(d, d);
          pin_order();
          for (int i0 = 0; i0 < n_tiles; i0 += kRingTK) {
#pragma unroll
            for (int d = 0; d < kRingTK; ++d) {
              const int i = i0 + d;
              if (i < n_tiles) {
                const int tile = tile_of(i);
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                  const v4f z = {0.f, 0.f, 0.f, 0.f};
                  v4f cx = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[0], kt[d][2 * u], z, 0, 0, 0);
                  v4f cy = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[1], kt[d][2 * u], z, 0, 0, 0);
                  cx = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[2], kt[d][2 * u + 1], cx, 0, 0, 0);
                  cy = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[3], kt[d][2 * u + 1], cy, 0, 0, 0);
                  v4f c;
#pragma unroll
                  for (int r = 0; r < 4; ++r) c[r] = cx[r] + dpp_f32<0x128>(cy[r]);     // row_ror 8
                  const int tok = tile * 16 + 8 * u + tsub;
                  // result rows 4 kb + r are heads: rows of lanes kb < NS hold the heads that exist
                  if (kb < NS && hsel == 0 && tok < ntx) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                      if (4 * kb + r < a.g) {
                        const float sv = c[r] * a.softmax_scale;
                        tlog[(4 * kb + r) * a.tstride + tok] = sv;
                        tmax[r] = fmaxf(tmax[r], sv);
                      }
                    }
                  }
                }
              }
              pin_order();
              load_tile(d, i + kRingTK);
              pin_order();
            }
          }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) tmax[r] = row_max(tmax[r]);
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
          for (int r = 0; r < 4; ++r) mref[4 * s + r] = lane_value(tmax[r], 16 * s);
        lds_publish();                           // the wave's logits before it reads them back
        // -- values of the wave's own shares
        if (n_own > 0) {
          float c2t[NH];
#pragma unroll
          for (int h = 0; h < NH; ++h) c2t[h] = -mref[h] * kLog2e;
          const __amdgpu_buffer_rsrc_t vt_buf =
              stream_buffer(a.v_text + ((size_t)row * a.n_text_cap + txt0) * kD, (unsigned)ntx * kD * 2);
          const int vt_lane = (kb * kD + 8 * n16) * 2;
          v4f acc_hi[NS][2], acc_lo[NS][2];      // [set][channel 8 n16 + 2 kb + i][head]
#pragma unroll
          for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int i = 0; i < 2; ++i) acc_hi[s][i] = acc_lo[s][i] = (v4f){0.f, 0.f, 0.f, 0.f};
          constexpr int kSteps = SH / 4, kDepth = kRingTV < kSteps ? kRingTV : kSteps, kRecs = SH / 16;
          static_assert(kSteps % kDepth == 0, "the ring divides a share");
          const int rec_wr = (((lane >> 2) / kRecs) * a.tstride) * 4 + ((lane >> 2) % kRecs) * 64 + (lane & 3) * 2;
          const int rec_rd = (lane & 3) * 8;     // matrix row = lane % 4 = head of the set
          v8h ring[kDepth];
          auto load_step = [&](int slot, int sh, int st) {
            ring[slot] = buffer_load_v8h<true>(vt_buf, vt_lane, (sh * SH + 4 * st) * (kD * 2));
          };
#pragma unroll
          for (int st = 0; st < kDepth; ++st) load_step(st, tw, st);
          pin_order();
          for (int sh = tw; sh < n_sh; sh += kBTextWaves) {
            const int t0 = sh * SH;
            const int nt = min(SH, ntx - t0);
            v4f pv[NS];
#pragma unroll
            for (int s = 0; s < NS; ++s) {
              pv[s] = (v4f){0.f, 0.f, 0.f, 0.f};
              if (lane < nt) {
#pragma unroll
                for (int j = 0; j < kHeads; ++j)
                  if (4 * s + j < a.g)
                    pv[s][j] = __builtin_amdgcn_exp2f(fmaf(tlog[(4 * s + j) * a.tstride + t0 + lane], kLog2e, c2t[4 * s + j]));
              }
#pragma unroll
              for (int j = 0; j < kHeads; ++j) lsum[4 * s + j] += pv[s][j];
            }
            uint8_t* pb = tbytes + (size_t)t0 * 4;
            __builtin_amdgcn_wave_barrier();
            asm volatile("" ::: "memory");       // the records overwrite logits read just above
            if (lane < SH) {                     // zero beyond nt
#pragma unroll
              for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int j = 0; j < kHeads; ++j) {
                  const float ps = pv[s][j] * 1024.f;
                  const _Float16 hi = (_Float16)ps;
                  const _Float16 lo = (_Float16)((ps - (float)hi) * 2048.f);
                  uint8_t* rec = pb + (size_t)(4 * s) * a.tstride * 4 + rec_wr + 8 * j;
                  *reinterpret_cast<_Float16*>(rec) = hi;
                  *reinterpret_cast<_Float16*>(rec + 32) = lo;
                }
            }
            lds_publish();
#pragma unroll
            for (int st = 0; st < kSteps; ++st) {
              const int slot = st % kDepth;
              const v4u32 raw = __builtin_bit_cast(v4u32, ring[slot]);
              const v2u lo2 = __builtin_amdgcn_permlane32_swap(raw[0], raw[2], false, false);
              const v2u hi2 = __builtin_amdgcn_permlane32_swap(raw[1], raw[3], false, false);
              const v2u t01 = __builtin_amdgcn_permlane16_swap(lo2[0], hi2[0], false, false);
              const v2u t23 = __builtin_amdgcn_permlane16_swap(lo2[1], hi2[1], false, false);
              const v2u even = {__builtin_amdgcn_perm(t01[1], t01[0], 0x05040100u),
                                __builtin_amdgcn_perm(t23[1], t23[0], 0x05040100u)};
              const v2u odd = {__builtin_amdgcn_perm(t01[1], t01[0], 0x07060302u),
                               __builtin_amdgcn_perm(t23[1], t23[0], 0x07060302u)};
              const v4h v_even = __builtin_bit_cast(v4h, even), v_odd = __builtin_bit_cast(v4h, odd);
#pragma unroll
              for (int s = 0; s < NS; ++s) {
                const uint8_t* rec = pb + (size_t)(4 * s + st / kRecs) * a.tstride * 4 + (st % kRecs) * 64 + rec_rd;
                const v4h p_hi = *reinterpret_cast<const v4h*>(rec);
                const v4h p_lo = *reinterpret_cast<const v4h*>(rec + 32);
                acc_hi[s][0] = __builtin_amdgcn_mfma_f32_4x4x4f16(p_hi, v_even, acc_hi[s][0], 0, 0, 0);
                acc_hi[s][1] = __builtin_amdgcn_mfma_f32_4x4x4f16(p_hi, v_odd, acc_hi[s][1], 0, 0, 0);
                acc_lo[s][0] = __builtin_amdgcn_mfma_f32_4x4x4f16(p_lo, v_even, acc_lo[s][0], 0, 0, 0);
                acc_lo[s][1] = __builtin_amdgcn_mfma_f32_4x4x4f16(p_lo, v_odd, acc_lo[s][1], 0, 0, 0);
              }
              if (st + kDepth < kSteps) load_step(slot, sh, st + kDepth);
              else load_step(slot, sh + kBTextWaves, st + kDepth - kSteps);
              pin_order();
            }
          }
          // lane (kb, n16): heads 0..3 of each set, channels 8 n16 + 2 kb and + 1
#pragma unroll
          for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int j = 0; j < kHeads; ++j) {
              const v2f pair = {fmaf(acc_lo[s][0][j], 0x1p-11f, acc_hi[s][0][j]) * 0x1p-10f,
                                fmaf(acc_lo[s][1][j], 0x1p-11f, acc_hi[s][1][j]) * 0x1p-10f};
              *reinterpret_cast<v2f*>(partial + (4 * s + j) * kD + 8 * n16 + 2 * kb) = pair;
            }
        }
      };
      const int rounds64 = ((ntx + 63) / 64 + kBTextWaves - 1) / kBTextWaves;
      const int rounds16 = ((ntx + 15) / 16 + kBTextWaves - 1) / kBTextWaves;
      if (11 * rounds16 < 40 * rounds64) text_part(std::integral_constant<int, 16>{});
      else text_part(std::integral_constant<int, 64>{});
    }
  }
  // a wave without tokens (a chunk of fewer tiles than visual waves, no text in the chunk, fewer
  // shares than text waves) has l = 0 and a reference point of -FLT_MAX; its partial sums get
  // weight 0 in the merge, but must be finite
  if (!wrote) {
    for (int i = lane; i < NH * kD; i += 64) partial[i] = 0.f;
  }
  // per-wave sums of the weights and of the additive value term (sum_j p_j min_j), per head
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    const float l = wave_sum(lsum[h]), m = wave_sum(msum[h]);
    if (lane == 0) {
      if (!vis_wave) mla[(wave * NH + h) * 3 + 0] = wrote ? mref[h] : -FLT_MAX;
      mla[(wave * NH + h) * 3 + 1] = l;
      mla[(wave * NH + h) * 3 + 2] = m;
    }
  }
  __syncthreads();

  // ---- epilogue: merge the waves (each with its own reference point) into one partial of the
  // joint softmax per head for the combine kernel
  const float* part_all = tlog + (size_t)NH * a.tstride;
  for (int e = tid; e < NH * kD; e += kBThreads) {
    const int h = e >> 7, c = e & 127;
    if (h < a.g) {
      float M = -FLT_MAX;
#pragma unroll
      for (int wv = 0; wv < kBWaves; ++wv) M = fmaxf(M, mla[(wv * NH + h) * 3]);
      float num = 0.f, den = 0.f;
#pragma unroll
      for (int wv = 0; wv < kBWaves; ++wv) {
        const float* r = mla + (wv * NH + h) * 3;
        const float wgt = __builtin_amdgcn_exp2f((r[0] - M) * kLog2e);    // 0 for a wave without tokens
        num = fmaf(wgt, part_all[((size_t)wv * NH + h) * kD + c] + r[2], num);
        den = fmaf(wgt, r[1], den);
      }
      float* out = a.ws_partial + ((head0 + h) * n_slots + slot) * (size_t)(kD + 2);
      if (c == 0) { out[0] = M; out[1] = den; }
      out[2 + c] = num;
    }
  }
}

size_t stream_values_lds(int ns, int tstride) {
  const size_t nh = (size_t)ns * kHeads;
  return (size_t)kBVisWaves * (ns * 1024 + 2048) + nh * tstride * 4 + (size_t)kBWaves * nh * kD * 4 +
         (size_t)kBWaves * nh * 3 * 4;
}
size_t stream_values_lds(int ns, int tstride, int ref_stride) {
  return stream_values_lds(ns, tstride) + (size_t)ns * kHeads * ref_stride * 4;
}
size_t stream_logits_lds(int ns) {
  return (size_t)ns * kHeads * kD * 4 + (size_t)kAWaves * ns * 2048 + (size_t)2 * ns * kAWaves * 4 +
         (size_t)kAWaves * ns * kHeads * 2 * 4;
}

constexpr int kMaxDevices = 64;
long long cu_count() {
  static std::atomic<int> n_cus[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int v = n_cus[dev].load(std::memory_order_relaxed);
  if (v == 0) {
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
      return 256;
    n_cus[dev].store(v, std::memory_order_relaxed);
  }
  return v;
}

}  // namespace

StreamPlan make_stream_plan(const DecodeShape& s, int min_chunks) {
  StreamPlan p;
  if (s.d != kD || (s.bits != 1 && s.bits != 2)) return p;
  if (s.k_axis != CQ_AXIS_CHANNEL || s.k_group != 128 || s.n_vis < 128 || s.n_vis % 128 != 0) return p;
  if (s.v_axis != CQ_AXIS_TOKEN || s.v_group != kD) return p;
  if (s.g < 1 || s.g > 2 * kHeads) return p;
  const long long rows = (long long)s.B * s.Hkv;
  const long long cus = cu_count();
  const int n_groups = s.n_vis / 128;
  auto clamp = [](long long v, long long lo, long long hi) { return (int)(v < lo ? lo : v > hi ? hi : v); };
  // logits pass: workgroups of 4 waves, three of them resident per CU with two head sets (the
  // registers of 3 waves per SIMD), four with one; chunks of at least 8 key groups (2 per wave)
  const long long wg_per_cu = s.g > kHeads ? 3 : 4;
  p.ca = clamp((wg_per_cu * cus + rows - 1) / rows, 1, n_groups >= 8 ? n_groups / 8 : 1);
  // values pass: workgroups of 4 waves, as many resident per CU as in the logits pass (two-bit
  // codes with the sets split over the waves would fit four as well and are 5 % slower that way:
  // 110 against 105 us on the long-context configuration); chunks of at least 8 groups (2 per
  // wave).  The fp16 tail goes out in chunks of at least four 64-token blocks (one per wave): a
  // text wave is slow on its own (one stream of loads), so its workgroups must be short.
  p.cb = clamp((wg_per_cu * cus + rows - 1) / rows, 1, n_groups >= 8 ? n_groups / 8 : 1);
  const int n_tblocks = (s.n_text + 63) / 64;
  p.ct = n_tblocks == 0 ? 0 : clamp(n_tblocks / 4, 1, 16);
  if (p.ca > 64) p.ca = 64;
  if (p.cb > 64) p.cb = 64;
  if (min_chunks > 1) {                          // a test's override: at least that many in both passes
    if (p.ca < min_chunks) p.ca = min_chunks < n_groups ? min_chunks : n_groups;
    if (p.cb < min_chunks) p.cb = min_chunks < n_groups ? min_chunks : n_groups;
  }
  const size_t heads = (size_t)s.B * s.Hq;
  auto align64 = [](size_t x) { return (x + 63) / 64 * 64; };
  // the buffer descriptors of the logits pass address a row's heads with 32-bit byte offsets
  if ((size_t)s.g * s.n_vis * 2 >= ((size_t)1 << 31)) return p;
  p.ws_lref_floats = align64(heads * p.ca * 2);
  p.ws_logits_floats = align64(p.ws_lref_floats + heads * (size_t)(s.n_vis / 128));
  p.ws_partial_floats = align64(p.ws_logits_floats + (heads * (size_t)s.n_vis + 1) / 2);
  const size_t floats = p.ws_partial_floats + heads * (size_t)(p.cb + p.ct) * (kD + 2);
  p.ws_bytes = (floats * sizeof(float) + 255) / 256 * 256;
  p.ok = true;
  return p;
}

hipError_t launch_decode_stream(const DecodeShape& s, const StreamPlan& plan, const void* q,
                                const cq_qtensor_t& k, const cq_qtensor_t& v, const void* k_text,
                                const void* v_text, const int32_t* n_text_dev, const Calib& calib,
                                float softmax_scale, void* out, float* workspace,
                                hipStream_t stream) {
  if (!plan.ok) return hipErrorInvalidValue;
  StreamArgs a;
  a.q = static_cast<const __half*>(q);
  a.k_codes = k.codes; a.k_scale = k.scale; a.k_min = k.min;
  a.v_codes = v.codes; a.v_scale = v.scale; a.v_min = v.min;
  a.k_text = static_cast<const __half*>(k_text);
  a.v_text = static_cast<const __half*>(v_text);
  a.g = s.g; a.n_vis = s.n_vis; a.n_text = s.n_text; a.n_text_cap = s.n_text_cap;
  a.n_text_dev = n_text_dev;
  const int n_groups = s.n_vis / 128, n_tblocks = (s.n_text + 63) / 64;
  auto magic = [](int c) { return c == 1 ? 0u : (unsigned)((((unsigned long long)1 << 32) / (unsigned)c) + 1); };
  a.ca = plan.ca; a.ca_base = n_groups / plan.ca; a.ca_rem = n_groups % plan.ca; a.ca_magic = magic(plan.ca);
  a.cb = plan.cb; a.cb_base = n_groups / plan.cb; a.cb_rem = n_groups % plan.cb; a.cb_magic = magic(plan.cb);
  a.ct = plan.ct; a.ct_magic = plan.ct > 0 ? magic(plan.ct) : 0u;
  a.tb_base = plan.ct > 0 ? n_tblocks / plan.ct : 0; a.tb_rem = plan.ct > 0 ? n_tblocks % plan.ct : 0;
  // text slots of a chunk: whole 64-token blocks; row pitch = 16 (mod 32) floats, conflict-free
  int tstride = (a.tb_base + (a.tb_rem ? 1 : 0)) * 64;
  tstride += (16 - (tstride % 32) + 32) % 32;
  a.tstride = tstride;
  a.ws_minmax = workspace;
  a.ws_lref = workspace + plan.ws_lref_floats;
  a.ws_logits = reinterpret_cast<uint16_t*>(workspace + plan.ws_logits_floats);
  // a falling calibration line known on the host: the smallest logits carry the largest weights
  a.falling = calib.mode == CQ_CALIB_FIXED && (calib.delta - calib.gamma + calib.tau1 - calib.tau2) < 0.f;
  a.ref_stride = n_groups / plan.cb + 1;         // key groups of the largest chunk of the values pass
  a.ws_partial = workspace + plan.ws_partial_floats;
  a.calib_mode = calib.mode; a.tau1 = calib.tau1; a.tau2 = calib.tau2;
  a.gamma = calib.gamma; a.delta = calib.delta; a.softmax_scale = softmax_scale;
  const size_t rows = (size_t)s.B * s.Hkv;
  const size_t blocks_a = rows * plan.ca, blocks_b = rows * (size_t)(plan.cb + plan.ct);
  a.n_text_wg = (int)(rows * plan.ct);
  // row = piece / chunks by multiplication: exact while piece * chunks < 2^32
  if (blocks_a * plan.ca >= ((size_t)1 << 32) || blocks_b * (plan.cb + plan.ct) >= ((size_t)1 << 32) ||
      blocks_a > 0x7fffffffu || blocks_b > 0x7fffffffu)
    return hipErrorInvalidConfiguration;
  const int ns = s.g > kHeads ? 2 : 1;
  const int hl = s.g - kHeads * (ns - 1);        // heads of the last set
  void (*kern_a)(const StreamArgs) = nullptr;
  void (*kern_b)(const StreamArgs) = nullptr;
  int slot = 0;
  auto values_kernel = [hl](auto bits, auto sets) -> void (*)(const StreamArgs) {
    constexpr int B = decltype(bits)::value, S = decltype(sets)::value;
    // two head sets per wave: one register slot for the packed values in flight (no spills, and
    // faster than two slots with spills at either code width)
    constexpr bool kOne = S == 2;
    switch (hl) {
      case 1: return stream_values_kernel<B, S, 1, kOne>;
      case 2: return stream_values_kernel<B, S, 2, kOne>;
      case 3: return stream_values_kernel<B, S, 3, kOne>;
      default: return stream_values_kernel<B, S, 4, kOne>;
    }
  };
  using std::integral_constant;
  switch (s.bits * 2 + ns) {
    case 1 * 2 + 1:
      kern_a = stream_logits_kernel<1, 1>;
      kern_b = values_kernel(integral_constant<int, 1>{}, integral_constant<int, 1>{});
      slot = 0;
      break;
    case 1 * 2 + 2:
      kern_a = stream_logits_kernel<1, 2>;
      kern_b = values_kernel(integral_constant<int, 1>{}, integral_constant<int, 2>{});
      slot = 4;
      break;
    case 2 * 2 + 1:
      kern_a = stream_logits_kernel<2, 1>;
      kern_b = values_kernel(integral_constant<int, 2>{}, integral_constant<int, 1>{});
      slot = 8;
      break;
    case 2 * 2 + 2:
      kern_a = stream_logits_kernel<2, 2>;
      kern_b = values_kernel(integral_constant<int, 2>{}, integral_constant<int, 2>{});
      slot = 12;
      break;
    default: return hipErrorInvalidValue;
  }
  slot += hl - 1;
  const size_t lds_a = stream_logits_lds(ns), lds_b = stream_values_lds(ns, tstride, a.ref_stride);
  if (lds_b > 160 * 1024) return hipErrorInvalidConfiguration;
  // the values kernel's dynamic LDS limit is raised once per (device, kernel) and only ever grows
  static std::atomic<size_t> configured[kMaxDevices][16];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (lds_b > 48 * 1024 && lds_b > configured[dev][slot].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern_b),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_b);
    if (e != hipSuccess) return e;
    size_t seen = configured[dev][slot].load(std::memory_order_relaxed);
    while (seen < lds_b &&
           !configured[dev][slot].compare_exchange_weak(seen, lds_b, std::memory_order_release)) {
    }
  }
  kern_a<<<dim3((unsigned)blocks_a), dim3(kAThreads), lds_a, stream>>>(a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  kern_b<<<dim3((unsigned)blocks_b), dim3(kBThreads), lds_b, stream>>>(a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_combine(s.B * s.Hq, plan.cb + plan.ct, kD, a.ws_partial, out, stream);
}

}  // namespace cq
