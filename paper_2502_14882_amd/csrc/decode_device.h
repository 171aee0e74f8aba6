// Device helpers shared by the tuned decode kernels (decode_fused.hip, decode_stream.hip): vector
// types, streaming loads, wave reductions on the DPP network, the fixed-point operand format of
// the int8 matrix-core contractions and the masks that turn packed codes into operands.
// Internal to libcq (not part of the ABI); everything is inline device code.
#ifndef CQ_DECODE_DEVICE_H_
#define CQ_DECODE_DEVICE_H_

#include <hip/hip_fp16.h>

#include <cfloat>
#include <stdint.h>

namespace cq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

constexpr int kD = 128;             // head_dim
constexpr int kHeads = 4;           // query heads per matrix pass (4 digits x 4 heads = 16 rows)
constexpr float kLog2e = 1.4426950408889634f;

// First unit of chunk c when n = base * n_chunks + rem units are dealt to n_chunks chunks, the
// first rem of them taking base + 1 (host and device share the rule).
__host__ __device__ inline int chunk_first(int base, int rem, int c) { return c * base + (c < rem ? c : rem); }


// Load of cache data that the workgroup reads exactly once.  NT marks it non-temporal (measured on
// a plain streaming read of the same bytes: 6.4-6.6 TB/s against 5.8 TB/s with ordinary loads).
// That only pays where one instruction covers whole cache lines: a line that several instructions
// touch in turn (the strided code words of 4- and 8-bit tokens) may be dropped in between and
// fetched again, so those loads stay ordinary, and so do all loads of a workgroup whose twin on
// the same XCD is meant to find the lines in L2 (two head blocks per KV head).
template <bool NT, typename T>
__device__ inline T stream_load(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}

// Streaming load through a buffer descriptor: the address is descriptor base + a per-lane offset
// that never changes + a wave-uniform offset in a scalar register, so a load costs no vector
// instruction for its address, and a read beyond the descriptor's size returns zeros instead of
// needing a clamped index.
typedef unsigned int v4u32 __attribute__((ext_vector_type(4)));
__device__ inline __amdgpu_buffer_rsrc_t stream_buffer(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
template <bool NT>
__device__ inline v8h buffer_load_v8h(__amdgpu_buffer_rsrc_t r, int lane_offset, int wave_offset) {
  return __builtin_bit_cast(v8h, __builtin_amdgcn_raw_buffer_load_b128(r, lane_offset, wave_offset, NT ? 2 : 0));
}

__device__ inline v2i lds_read_tr8(const uint8_t* p) {
  return __builtin_amdgcn_ds_read_tr8_b64_v2i32(
      (__attribute__((address_space(3))) v2i*)(p));
}

template <int CTRL> __device__ inline float dpp_f32(float v);
// Sum over the wave on the DPP network; the result is wave-uniform.
__device__ inline float wave_sum(float v) {
  v += dpp_f32<0xB1>(v);      // quad_perm 1,0,3,2
  v += dpp_f32<0x4E>(v);      // quad_perm 2,3,0,1: every lane holds its quad's sum
  v += dpp_f32<0x141>(v);     // row_half_mirror: the other quad of the half row
  v += dpp_f32<0x140>(v);     // row_mirror: the other half row
  const int r1 = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false);
  v += __builtin_bit_cast(float, r1);     // row_bcast15: rows 1, 3 add the row before them
  const int r2 = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false);
  v += __builtin_bit_cast(float, r2);     // row_bcast31: rows 2, 3 add rows 0 + 1
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
// Maximum over the wave of a non-negative float, on the DPP network (no LDS round trips); the
// result is wave-uniform.  Non-negative floats order like their bit patterns.
__device__ inline float wave_max_nonneg(float v) {
  int x = __builtin_bit_cast(int, v);
  x = max(x, __builtin_amdgcn_update_dpp(x, x, 0xB1, 0xF, 0xF, true));    // quad_perm 1,0,3,2
  x = max(x, __builtin_amdgcn_update_dpp(x, x, 0x4E, 0xF, 0xF, true));    // quad_perm 2,3,0,1
  x = max(x, __builtin_amdgcn_update_dpp(x, x, 0x141, 0xF, 0xF, true));   // row_half_mirror
  x = max(x, __builtin_amdgcn_update_dpp(x, x, 0x140, 0xF, 0xF, true));   // row_mirror
  x = max(x, __builtin_amdgcn_update_dpp(x, x, 0x142, 0xA, 0xF, false));  // row_bcast15 -> rows 1,3
  x = max(x, __builtin_amdgcn_update_dpp(x, x, 0x143, 0xC, 0xF, false));  // row_bcast31 -> rows 2,3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(x, 63));
}
// value of four signed base-256 digit accumulators
__device__ inline float digits_to_float(const v4i& c) {
  return fmaf(fmaf(fmaf((float)c[3], 256.f, (float)c[2]), 256.f, (float)c[1]), 256.f, (float)c[0]);
}
// Keeps the software pipelines as written: without it the compiler moves a ring's loads across the
// loop back-edge next to their use, which exposes the full memory latency in every iteration.
__device__ inline void pin_order() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}
__device__ inline void lds_publish() {   // this wave's LDS writes before its later LDS reads
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

template <int CTRL>
__device__ inline float dpp_f32(float v) {
  const int x = __builtin_bit_cast(int, v);
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, true));
}

// Reductions over the 16 lanes of a row of the wave, on the DPP network; every lane of the row
// ends up with the row's result.
__device__ inline float row_min(float v) {
  v = fminf(v, dpp_f32<0xB1>(v));     // quad_perm 1,0,3,2
  v = fminf(v, dpp_f32<0x4E>(v));     // quad_perm 2,3,0,1
  v = fminf(v, dpp_f32<0x141>(v));    // row_half_mirror
  return fminf(v, dpp_f32<0x140>(v)); // row_mirror
}
__device__ inline float row_max(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));
  v = fmaxf(v, dpp_f32<0x4E>(v));
  v = fmaxf(v, dpp_f32<0x141>(v));
  return fmaxf(v, dpp_f32<0x140>(v));
}
__device__ inline float row_sum(float v) {
  v += dpp_f32<0xB1>(v);
  v += dpp_f32<0x4E>(v);
  v += dpp_f32<0x141>(v);
  return v + dpp_f32<0x140>(v);
}
__device__ inline float lane_value(float v, int lane) {     // wave-uniform copy of one lane's value
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// Additive post-scaling term of one key group, sum_c q'[h][c] * min[c] for the four heads.  Every
// lane brings two channels (q' already carries the softmax scale and the lane's operand weight
// w, which inv_w = 1/w takes out again, per channel).  A transposing butterfly leaves lane (.., b1, b0) with head
// 2*b0 + b1 after two steps, the remaining steps add lanes that hold the same head; the result
// lane of head kb = lane / 16 then fetches its head.
// off0/off1: what the operand bytes leave out per channel (128 * scale for 8-bit codes, else 0).
__device__ inline float group_bias(const float (&qv0)[kHeads], const float (&qv1)[kHeads],
                                   uint16_t m0, uint16_t m1, float off0, float off1, float inv_w0,
                                   float inv_w1, int lane) {
  const float f0 = (__half2float(__ushort_as_half(m0)) + off0) * inv_w0;
  const float f1 = (__half2float(__ushort_as_half(m1)) + off1) * inv_w1;
  float part[kHeads];
#pragma unroll
  for (int h = 0; h < kHeads; ++h) part[h] = fmaf(qv0[h], f0, qv1[h] * f1);
  const bool b0 = lane & 1, b1 = lane & 2;
  float u0 = b0 ? part[2] : part[0], u1 = b0 ? part[3] : part[1];
  const float g0 = b0 ? part[0] : part[2], g1 = b0 ? part[1] : part[3];
  u0 += dpp_f32<0xB1>(g0);                 // quad_perm 1,0,3,2: lane ^ 1
  u1 += dpp_f32<0xB1>(g1);
  float r = b1 ? u1 : u0;
  const float g2 = b1 ? u0 : u1;
  r += dpp_f32<0x4E>(g2);                  // quad_perm 2,3,0,1: lane ^ 2
  r += dpp_f32<0x124>(r);                  // row_ror 4
  r += dpp_f32<0x128>(r);                  // row_ror 8
  // Every lane of a row now holds the row's sum for head bitrev2(lane & 3).  What is wanted is the
  // sum over the four rows, head kb in row kb: the four heads side by side (quad broadcasts), then
  // a transposing fold over the rows with paired lane swaps (a swap of two values and one add
  // halve both) - all on the vector unit, where this used to take three LDS round trips per group.
  const float h0 = dpp_f32<0x00>(r), h1 = dpp_f32<0xAA>(r);     // quad lanes 0 and 2
  const float h2 = dpp_f32<0x55>(r), h3 = dpp_f32<0xFF>(r);     // quad lanes 1 and 3
  auto bits_of = [](float v) { return __builtin_bit_cast(unsigned, v); };
  auto float_of = [](unsigned v) { return __builtin_bit_cast(float, v); };
  const auto e = __builtin_amdgcn_permlane32_swap(bits_of(h0), bits_of(h2), false, false);
  const auto o = __builtin_amdgcn_permlane32_swap(bits_of(h1), bits_of(h3), false, false);
  const float s02 = float_of(e[0]) + float_of(e[1]);            // head 0 in lanes 0-31, head 2 in 32-63
  const float s13 = float_of(o[0]) + float_of(o[1]);            // head 1 | head 3
  const auto t = __builtin_amdgcn_permlane16_swap(bits_of(s02), bits_of(s13), false, false);
  return float_of(t[0]) + float_of(t[1]);                       // rows 0..3: heads 0, 1, 2, 3
}

// Fixed-point operands are |x| < 2^29, four signed base-256 digits.  The wide range is needed
// because one shift serves a whole key group (or value tile): with heavy-tailed channel scales
// the ordinary channels sit 2^10 or more below the largest one and still need ~16 bits.  At
// this width truncation (one v_cvt) is as good as rounding: the bias it adds is below 2^-28 of
// the largest operand per term.
// Largest F with bound * 2^F <= 2^29, clamped so that 2^F and 2^-F stay normal floats.
__device__ inline int fixed_point_shift(float bound) {
  if (!(bound > 0.f)) return 90;
  int e;
  frexpf(bound, &e);           // bound = m * 2^e, m in [0.5, 1)
  return max(-90, min(90, 29 - e));
}
// the four signed base-256 digits of a * b (truncated), as the four bytes of the result:
// digits(x) = (x + 0x00808080) ^ 0x00808080, with the addition riding on the fma (the float sum is
// exact to one unit below 2^24 and to fp32 precision above, which is all the product has)
__device__ inline int product_digits(float a, float b) {
  return (int)fmaf(a, b, 8421504.f) ^ 0x00808080;
}

// Masks that turn a packed word into int8 operands, and what an operand byte is worth.  A byte
// of a word holds 8 / b codes; variant v picks code v of every byte (from the low bits up):
//   b = 1: v in 0..7, mask 0x01010101 << v, byte = bit * 2^v (-128 for v = 7)
//   b = 2: v in 0..3, masks 0x03 / 0x0c / 0x30 per byte and (word >> 2) & 0x30 for the top
//          code of each byte, byte = code * {1, 4, 16, 16}
//   b = 4: v in 0..1, word & 0x0f.. and (word >> 4) & 0x0f.., byte = code
//   b = 8: the byte is the code; word ^ 0x80.. is code - 128 as int8, and the 128 is added back
//          through the additive term (it multiplies the same scale)
template <int BITS>
__device__ inline int operand_variant(uint32_t word, int v) {
  if constexpr (BITS == 1) return (int)(word & (0x01010101u << v));
  else if constexpr (BITS == 2)
    return v < 3 ? (int)(word & (0x03030303u << (2 * v))) : (int)((word >> 2) & 0x30303030u);
  else if constexpr (BITS == 4) return (int)((v ? word >> 4 : word) & 0x0f0f0f0fu);
  else return (int)(word ^ 0x80808080u);
}
template <int BITS>
__device__ inline float variant_weight(int v) {     // 1 / (value of a set code-1 byte)
  if constexpr (BITS == 1) return ldexpf(1.f, -v) * (v == 7 ? -1.f : 1.f);
  else if constexpr (BITS == 2) return v == 0 ? 1.f : v == 1 ? 0.25f : 0.0625f;
  else return 1.f;
}
// Position, inside its 32-bit word, of the code that variant v reads from byte y: the packing is
// MSB first, so code j sits at bits [32 - b(1 + j), 32 - b j).
template <int BITS>
__device__ inline int code_in_word(int y, int v) {
  return (32 / BITS - 1) - ((8 / BITS) * y + v);
}

// TILES = 16-token tiles per key group (k_group / 16); BITS = code width (1, 2, 4 or 8); VCH = values

}  // namespace
}  // namespace cq

#endif  // CQ_DECODE_DEVICE_H_
