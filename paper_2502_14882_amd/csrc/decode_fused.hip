// Fused decode attention over the packed cache (1, 2, 4 or 8 bits) for head_dim 128 (gfx950).
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
//
// Work split inside the workgroup (12 waves): waves 0..7 stream the packed visual cache, waves
// 8..11 stream the fp16 text tail at the same time (its two contractions on the fp16 matrix cores:
// 16 x 16 x 32 for the logits, 4 x 4 x 4 blocks for the values), so the bandwidth-heavy text reads
// overlap the compute-heavy visual phases.  Every stream keeps a ring of loads several tiles deep in flight.
// Two rules keep those rings in flight (the compiler's wait counting is exact only in straight
// code): the steady-state loops have no branch around a global load (clamped addresses, tails
// apart, group ends known at compile time), and nothing keeps a loaded register alive past the
// ring's next load into it (values are converted when they are used first).  Broken, either rule
// costs an `s_waitcnt vmcnt(0)` per iteration.
#include <hip/hip_fp16.h>

#include <atomic>
#include <cfloat>
#include <type_traits>

#include "cq_internal.h"
#include "decode_device.h"

namespace cq {
namespace {


constexpr int kVisWaves = 8;        // waves on the packed visual cache
constexpr int kTextWaves = 4;       // waves on the fp16 text tail
constexpr int kWaves = kVisWaves + kTextWaves;
constexpr int kThreads = kWaves * 64;
constexpr int kStageBytes = 2048;   // LDS staging per visual wave
constexpr int kRedPerHead = 6;
// loads in flight per wave, in units of one key group / value tile / text tile / 4 text tokens.
// Deeper is not better on this chip: with much more in flight per CU the achieved bandwidth drops
// (also seen on a plain streaming read).  Measured: on long whole rows (64 key groups) 3 key
// groups in flight are 1-2 % faster than 2 and 4 are 8 % slower (about 1 % faster with groups of
// 32 tokens, slower with 64), on short or split rows 3 are 3-5 % slower (the kernel's RK
// parameter); the other rings make no difference.
constexpr int kRingK = 2, kRingV = 2, kRingT = 2, kRingTV = 4;
static_assert(kRingV % 2 == 0, "value tiles alternate between two LDS buffers");
// kModeFull: the workgroup owns the whole row and writes `out`.  A row that does not fit LDS, has
// more than 4 query heads per KV head, or belongs to a batch too small to fill the chip is split
// into chunks: kModeExtrema publishes the extrema of each chunk's visual logits (needed first
// for the dynamic calibration range), kModePartial recomputes the chunk's logits in LDS and
// writes one online-softmax partial per (head, chunk) for the combine kernel.
enum { kModeFull = 0, kModeExtrema = 1, kModePartial = 2 };

struct FusedArgs {
  const __half* q;
  const uint32_t* k_codes; const float* k_scale; const uint16_t* k_min;
  const uint32_t* v_codes; const float* v_scale; const uint16_t* v_min;
  const __half* k_text; const __half* v_text;
  __half* out;
  int Hq, Hkv, g, n_vis, n_text, n_text_cap;
  const int32_t* n_text_dev;   // NULL, or the tail length in device memory (n_text is then its bound)
  int k_group;       // tokens that are processed as one key group (32, 64 or 128)
  int v_group;       // channel-wise values: tokens processed as one value group (64 or 128)
  // Parameters (scale, min) of channel-wise tensors: elements per row, and elements between two
  // consecutive processing groups.  Statistics over the whole sequence (Sec. 3.1 as printed: one
  // pair per channel) are one parameter group per row that every processing group of 128
  // tokens reads again: pstride = 0.
  int k_prow, k_pstride, v_prow, v_pstride;
  int unit;          // chunk boundaries are multiples of unit key groups
  int stride;        // floats between the logit rows of two heads in LDS
  int mode, n_chunks, nhb;   // kMode*, chunks per row, blocks of 4 query heads per KV head
  int n_pieces;              // rows * n_chunks
  unsigned chunks_magic;     // fl(2^32 / n_chunks) + 1, or 0 when n_chunks == 1
  int units_base, units_rem;       // units of visual tokens per chunk: quotient and remainder
  int tblocks_base, tblocks_rem;   // 64-token text blocks per chunk, likewise
  float* ws_minmax;  // split rows: [B*Hq][n_chunks][2] extrema of the visual logits
  float* ws_partial; // split rows: [B*Hq][n_chunks][d + 2] partials (m, l, acc) for the combine
  int calib_mode; float tau1, tau2, gamma, delta, softmax_scale;
};


extern __shared__ __align__(16) uint8_t smem[];

// quantized channel-wise over groups of tokens (Sec. 3.1, the paper's own choice) instead of
// token-wise.
// KW = key statistics over the whole sequence: one parameter group per row, so the query operand,
// its shift and the additive term are formed once per wave instead of once per 128 tokens.
template <int TILES, int BITS, bool VCH, bool KW = false, bool NT = true, int RK = kRingK>
__global__ void __launch_bounds__(kThreads)
fused_row_kernel(const FusedArgs a) {
  // code words, see stream_load: a key instruction covers whole lines up to b = 4, a value
  // instruction up to b = 2 (wider value codes are read token by token in 16-byte pieces)
  constexpr bool kNtKeys = NT && BITS <= 4, kNtCodes = NT && BITS <= 2;
  static_assert(!KW || TILES == 8, "whole-sequence keys are processed 128 tokens at a time");
  // the wave index as a scalar: what depends on the wave's role then branches and counts on the
  // scalar unit (1.5 % of the whole kernel)
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // workgroup = (row = b * Hkv + kvh, block of 4 query heads, chunk of the row's tokens)
  // Workgroups are handed to the 8 XCDs round-robin.  With two head blocks per KV head, the two
  // workgroups that read the same (row, chunk) get block indices 8 apart: same XCD, started
  // together, so the second one's key/value reads are served by that XCD's L2.
  // None of this divides: a division by a value that is only known at run time is emulated with
  // dozens of scalar instructions and several round trips through the vector unit, and the eight of
  // them that stood here ran (on every wave) before the first load of a workgroup could be issued.
  int piece = blockIdx.x, hb = 0;           // piece = row * n_chunks + chunk
  if (a.nhb > 1) {                          // nhb = 2: slot = block / 8, hb = slot % 2
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    hb = slot & 1;
    piece = (slot >> 1) * 8 + xcd;
    if (piece >= a.n_pieces) return;        // grid is rounded up to whole groups of 8 pieces
  }
  // row = piece / n_chunks by multiplication with the host's fl(2^32 / n_chunks) + 1 (exact while
  // piece * n_chunks < 2^32, which the host checks)
  const int row = a.chunks_magic ? (int)__umulhi((unsigned)piece, a.chunks_magic) : piece;
  const int chunk = piece - row * a.n_chunks;
  const int gh = min(kHeads, a.g - hb * kHeads);            // live query heads of this block
  const size_t head0 = (size_t)row * a.g + (size_t)hb * kHeads;   // Hq = Hkv * g
  // the chunk's share of the visual tokens (whole key groups and whole 64-token tiles) and of
  // the 64-token text blocks: the first `rem` chunks take one unit more than the others
  const int unit = a.unit;
  const int ga = chunk_first(a.units_base, a.units_rem, chunk) * unit;
  const int gb = chunk_first(a.units_base, a.units_rem, chunk + 1) * unit;
  const int n_groups = gb - ga, nv = n_groups * a.k_group, vis0 = ga * a.k_group;
  const int ba = chunk_first(a.tblocks_base, a.tblocks_rem, chunk);
  const int bb = chunk_first(a.tblocks_base, a.tblocks_rem, chunk + 1);
  const int txt0 = ba * 64;
  // the tail length: the host's value, or the device's clamped to it (a growing tail in a replayed graph)
  const int n_text = a.n_text_dev ? min(max(*a.n_text_dev, 0), a.n_text) : a.n_text;
  const int ntx = a.mode == kModeExtrema ? 0 : max(0, min(n_text, bb * 64) - txt0);
  const bool vis_wave = wave < kVisWaves;
  const int tw = wave - kVisWaves;            // index among the text waves
  const int n16 = lane & 15, kb = lane >> 4;

  // ---- LDS carve-up
  float* logits = reinterpret_cast<float*>(smem);                       // [kHeads][stride]
  uint8_t* lbytes = smem;
  size_t off = (size_t)kHeads * a.stride * sizeof(float);
  if (off < (size_t)kWaves * kHeads * kD * sizeof(float)) off = (size_t)kWaves * kHeads * kD * sizeof(float);
  float* qf = reinterpret_cast<float*>(smem + off);   off += kHeads * kD * sizeof(float);
  off = (off + 15) & ~(size_t)15;
  uint8_t* stage = smem + off + (size_t)(vis_wave ? wave : 0) * kStageBytes;
  off += (size_t)kVisWaves * kStageBytes;
  float* red = reinterpret_cast<float*>(smem + off);   // [kWaves][kHeads][kRedPerHead]

  // rows of unused heads (g < 4) are computed along but never output; keep them finite.  Their
  // visual slots are written in phase 1 like everyone's (their query is zero, so are their
  // logits); only the text slots and the padding behind them are never written by anyone.
  for (int h = gh; h < kHeads; ++h)
    for (int i = nv + tid; i < a.stride; i += kThreads) logits[h * a.stride + i] = 0.f;

  // ---- phase 0: query to LDS and max |q| per head.  The fixed-point shifts and the additive
  // post-scaling term q . min_t are formed on the fly in phases 1 and 2 from the scales and minima
  // that the streaming loads bring in anyway, so every parameter is read exactly once.
  const float* ks_row = a.k_scale + (size_t)row * a.k_prow + (size_t)ga * a.k_pstride;
  const uint16_t* km_row = a.k_min + (size_t)row * a.k_prow + (size_t)ga * a.k_pstride;
  const float* vs_row = a.v_scale + (size_t)row * a.n_vis + vis0;
  const uint16_t* vm_row = a.v_min + (size_t)row * a.n_vis + vis0;
  if (tid < kHeads * kD) {
    const int h = tid / kD, c = tid % kD;
    const float qv = h < gh ? __half2float(a.q[(head0 + h) * kD + c]) : 0.f;
    qf[tid] = qv;
    const float m = wave_max_nonneg(fabsf(qv));     // waves 2h, 2h+1 hold head h
    if (lane == 0) red[wave] = m;
  }
  __syncthreads();
  float qmax[kHeads];
#pragma unroll
  for (int h = 0; h < kHeads; ++h) qmax[h] = fmaxf(red[2 * h], red[2 * h + 1]) * a.softmax_scale;
  const float qmax_all = fmaxf(fmaxf(qmax[0], qmax[1]), fmaxf(qmax[2], qmax[3]));
  __syncthreads();   // red is reused below
  // Split row: the chunk extrema of the first pass, which phase 2 needs for the calibration line,
  // are asked for here and arrive during phase 1 (lane 16h + w: head h, chunk w; a lane beyond the
  // live heads or chunks reads a neighbour's pair, which folds in harmlessly or is never used).
  v2f chunk_mm = {FLT_MAX, -FLT_MAX};
  if (a.mode == kModePartial && a.calib_mode == CQ_CALIB_DYNAMIC)
    chunk_mm = *reinterpret_cast<const v2f*>(
        a.ws_minmax + ((head0 + min(lane >> 4, gh - 1)) * a.n_chunks + min(lane & 15, a.n_chunks - 1)) * 2);

  // ring of the first value tiles of the narrow token-wise path (b <= 2): asked for during
  // phase 1, right after the first key groups, so that phase 2 does not start on a cold load
  constexpr bool kPrimeValues = !VCH && BITS <= 2;
  v4i p2_cg[kRingV][BITS];
  float p2_vsr[kRingV];
  uint16_t p2_vmr[kRingV];       // raw fp16 bits: converting here would wait for the load at once
  const uint32_t* p2_vc_row = a.v_codes + ((size_t)row * a.n_vis + vis0) * (4 * BITS);
  auto p2_load_tile = [&](int slot, int jt) {
    const int j0 = min(jt, nv - 64), j = j0 + lane;
    // the tile's code bytes are contiguous: instruction e takes the e-th KB, whole cache lines
#pragma unroll
    for (int e = 0; e < BITS; ++e)
      p2_cg[slot][e] = stream_load<kNtCodes>(reinterpret_cast<const v4i*>(p2_vc_row + (size_t)j0 * (4 * BITS) + 256 * e + 4 * lane));
    p2_vsr[slot] = stream_load<NT>(vs_row + j);
    p2_vmr[slot] = stream_load<NT>(vm_row + j);
  };

  // =================================================================== phase 1: logits
  if (vis_wave) {
    // Lane roles on a visual wave:
    //   writer of the query operand: lane handles two 16-byte LDS rows (two channels, all heads)
    //   matrix lane (n16, kb): token n16 of a 16-token tile, word kb of it
    //   result lane: token n16, head kb (its four digits are the lane's four accumulators)
    const int hres = kb;
    float mn = FLT_MAX, mx = -FLT_MAX;
    if (nv > 0) {
      // operand rows: r = ((kb*2 + i)*4 + v)*4 + y, i = matrix, v = register, y = byte.  Lane
      // (n16, kb) holds words kb*b .. kb*b + b-1 of its token = channels 32kb .. 32kb + 31:
      //   b = 1: row r <-> channel 32kb + 31 - (4i+v) - 8y, mask variant 4i + v;
      //   b = 2: matrix i takes word 2kb + i; row r <-> channel 32kb + 16i + 15 - 4y - v;
      //   b = 4: matrix i takes words 4kb + 2i, +1, two variants each; b = 8: words 8kb + 4i .. +3.
      // Row r lives at base + (r / 32) * pitch + (r % 32) * 16.
      // register v of matrix i is pair 4i + v of the lane's 8 (word, variant) pairs:
      // word (4i + v) / (8/b) of the lane's b words, variant (4i + v) % (8/b).
      // Writing the rows is a job of its own: lane (kb, l) writes the rows of the two ADJACENT
      // channels 32kb + 2l and + 1, so that their scales (one 8-byte load) and minima (one 4-byte
      // load) come in fully coalesced; which rows those are follows from inverting the map above.
      constexpr int kV = 8 / BITS, kCW = 32 / BITS;       // variants per byte, codes per word
      const int wc0 = 32 * kb + 2 * n16, wc1 = wc0 + 1;
      auto row_of = [&](int c, int& variant) {            // row inside the kb block, and its variant
        const int cl = c & 31, e = cl / kCW, t = kCW - 1 - cl % kCW;
        const int y = t / kV, v = t % kV, pair = e * kV + v;
        variant = v;
        return pair * 4 + y;
      };
      int wvar0, wvar1;
      const int wr0 = row_of(wc0, wvar0), wr1 = row_of(wc1, wvar1);
      float qv0[kHeads], qv1[kHeads];               // set below, behind the first loads
      const float inv_w0 = 1.f / variant_weight<BITS>(wvar0);   // exact: powers of two
      const float inv_w1 = 1.f / variant_weight<BITS>(wvar1);
      const uint32_t* kc_lane =
          a.k_codes + ((size_t)row * a.n_vis + vis0) * (4 * BITS) + n16 * (4 * BITS) + kb * BITS;
      float* lrow = logits + (size_t)hres * a.stride + n16;
      // with 128-token groups the operand rows of a group are staged in the group's own logit
      // slots (2 KB, not yet written); smaller groups use the wave's staging buffer
      constexpr bool kInPlace = (TILES == 8) && !KW;
      const int pitch = kInPlace ? a.stride * 4 : 512;
      const int x_wr0 = kb * pitch + wr0 * 16, x_wr1 = kb * pitch + wr1 * 16;
      const int x_rd = kb * pitch + (n16 >> 1) * 16 + (n16 & 1) * 8;

      // wide codes are 4 or 8 words per lane and tile: one group in the ring is all that fits
      // (the depth of this ring was measured to make no difference)
      constexpr int kRK = BITS > 2 ? 1 : RK;
      // One-bit keys are read 16 bytes per lane: a wave-wide load is then four whole tiles (1 KB in
      // one piece) instead of one tile's 256 bytes, which the memory pipeline serves ~12 % faster
      // (measured with the loads of this phase alone).  Lane (n16, kb) reads all four words of
      // token n16 of tile 4j + kb; a 4 x 4 transpose over the wave's four rows of lanes, two lane
      // swaps per register pair, leaves it with word kb of tiles 4j .. 4j + 3, which is what the
      // matrix operand wants.  The transpose is done when the group is used, not when it is loaded.
      constexpr bool kQuadKeys = BITS == 1 && TILES % 4 == 0;
      constexpr int kQuads = kQuadKeys ? TILES / 4 : 1;
      uint32_t w[kQuadKeys ? 1 : kRK][TILES][BITS];
      v4i wq[kQuadKeys ? kRK : 1][kQuads];
      const uint32_t* kq_lane =
          a.k_codes + ((size_t)row * a.n_vis + vis0) * 4 + (size_t)(16 * kb + n16) * 4;
      v2f s01[kRK];               // scales of channels wc0, wc1
      uint32_t m01[kRK];          // their minima, two fp16 in one word
      auto load_group = [&](int slot, int t) {
        const int tc = min(t, n_groups - 1);      // clamped, never a branch around a load
        // a lane's b words of a tile are adjacent: one load of 4b bytes (two of 16 for b = 8), so
        // that an instruction covers whole cache lines
        if constexpr (kQuadKeys) {
#pragma unroll
          for (int j = 0; j < kQuads; ++j)
            wq[slot][j] = stream_load<kNtKeys>(
                reinterpret_cast<const v4i*>(kq_lane + ((size_t)tc * TILES + 4 * j) * 64));
        }
#pragma unroll
        for (int i = 0; i < (kQuadKeys ? 0 : TILES); ++i) {
          const uint32_t* p = kc_lane + ((size_t)tc * TILES + i) * (64 * BITS);
          if constexpr (BITS == 1) {
            w[slot][i][0] = stream_load<kNtKeys>(p);
          } else if constexpr (BITS == 2) {
            const v2i t2 = stream_load<kNtKeys>(reinterpret_cast<const v2i*>(p));
            w[slot][i][0] = (uint32_t)t2[0];
            w[slot][i][1] = (uint32_t)t2[1];
          } else {
#pragma unroll
            for (int q4 = 0; q4 < BITS / 4; ++q4) {
              const v4i t4 = stream_load<kNtKeys>(reinterpret_cast<const v4i*>(p) + q4);
#pragma unroll
              for (int u = 0; u < 4; ++u) w[slot][i][4 * q4 + u] = (uint32_t)t4[u];
            }
          }
        }
        if constexpr (!KW) {
          s01[slot] = stream_load<NT>(reinterpret_cast<const v2f*>(ks_row + (size_t)tc * a.k_pstride + wc0));
          m01[slot] = stream_load<NT>(reinterpret_cast<const uint32_t*>(km_row + (size_t)tc * a.k_pstride + wc0));
        }
      };
      // query operand of the key group whose parameters sit in ring slot `slot`, staged at xb
      auto build_operand = [&](int slot, uint8_t* xb, v4i& A0, v4i& A1, float& bias_h,
                               float& inv_f, float& inv_f16) {
        // |q'| <= max|q| * (largest scale of the group): a bound, good to a few bits, that costs
        // one wave-wide maximum instead of a pass over all scales
        const float s0 = s01[slot][0], s1 = s01[slot][1];
        const float smax = wave_max_nonneg(fmaxf(s0, s1));
        const int F = fixed_point_shift(qmax_all * smax);      // one shift for the four heads
        const float s0f = ldexpf(s0, F), s1f = ldexpf(s1, F);
        v4i x0, x1;
#pragma unroll
        for (int h = 0; h < kHeads; ++h) {
          x0[h] = product_digits(qv0[h], s0f);
          x1[h] = product_digits(qv1[h], s1f);
        }
        inv_f = ldexpf(1.f, -F);
        inv_f16 = ldexpf(1.f, 16 - F);
        __builtin_amdgcn_wave_barrier();
        *reinterpret_cast<v4i*>(xb + x_wr0) = x0;
        *reinterpret_cast<v4i*>(xb + x_wr1) = x1;
        lds_publish();
        // A operand of matrix i: rows (kb*2 + i)*16 .. +15, two transposing reads of 8 rows
        const uint8_t* xr = xb + x_rd;
        const v2i r00 = lds_read_tr8(xr), r01 = lds_read_tr8(xr + 128);
        const v2i r10 = lds_read_tr8(xr + 256), r11 = lds_read_tr8(xr + 384);
        A0 = (v4i){r00[0], r00[1], r01[0], r01[1]};
        A1 = (v4i){r10[0], r10[1], r11[0], r11[1]};
        bias_h = group_bias(qv0, qv1, (uint16_t)(m01[slot] & 0xffffu), (uint16_t)(m01[slot] >> 16),
                                        BITS == 8 ? 128.f * s0 : 0.f, BITS == 8 ? 128.f * s1 : 0.f,
                                        inv_w0, inv_w1, lane);
        __builtin_amdgcn_wave_barrier();   // operand rows are consumed before logits land there
      };
      v4i A0w = {0, 0, 0, 0}, A1w = {0, 0, 0, 0};
      float bias_w = 0.f, inv_f_w = 0.f, inv_f16_w = 0.f;
      auto do_group = [&](int slot, int t) {
        v4i A0 = A0w, A1 = A1w;
        float bias_h = bias_w, inv_f = inv_f_w, inv_f16 = inv_f16_w;
        if constexpr (!KW)
          build_operand(slot, kInPlace ? lbytes + (size_t)t * (TILES * 16 * 4) : stage,
                        A0, A1, bias_h, inv_f, inv_f16);
        uint32_t wt[TILES];                         // one-bit keys: the lane's word of every tile
        if constexpr (kQuadKeys) {
#pragma unroll
          for (int j = 0; j < kQuads; ++j) {
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
        // the operands of tile + 1 are formed before the products of this tile are issued, so no
        // product waits on the ANDs right in front of it
        auto expand = [&](int tile, v4i& B0, v4i& B1) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            constexpr int kV = 8 / BITS;            // variants per byte
            if constexpr (kQuadKeys) {
              B0[v] = operand_variant<BITS>(wt[tile], v);
              B1[v] = operand_variant<BITS>(wt[tile], 4 + v);
            } else {
              B0[v] = operand_variant<BITS>(w[slot][tile][v / kV], v % kV);
              B1[v] = operand_variant<BITS>(w[slot][tile][(4 + v) / kV], (4 + v) % kV);
            }
          }
        };
        auto finish_tile = [&](int tile, const v4i& c) {
          const int lo = c[0] + (c[1] << 8), hi = c[2] + (c[3] << 8);
          const float sv = fmaf((float)hi, inv_f16, fmaf((float)lo, inv_f, bias_h));
          // lanes of unused heads (hres >= g) see q = 0, finish with sv = 0 and write their own
          // (never read) logit row: no branch in the hot loop
          lrow[(t * TILES + tile) * 16] = sv;
          mn = fminf(mn, sv);
          mx = fmaxf(mx, sv);
        };
        // two tiles at a time: their four products are interleaved so that the second product of
        // a tile (which accumulates onto the first) does not wait for it
        static_assert(TILES % 2 == 0, "tiles are taken in pairs");
#pragma unroll
        for (int tile = 0; tile < TILES; tile += 2) {
          v4i Ba0, Ba1, Bb0, Bb1;
          expand(tile, Ba0, Ba1);
          expand(tile + 1, Bb0, Bb1);
          __builtin_amdgcn_sched_barrier(0);
          v4i ca = {0, 0, 0, 0}, cb = {0, 0, 0, 0};
          ca = __builtin_amdgcn_mfma_i32_16x16x64_i8(A0, Ba0, ca, 0, 0, 0);
          cb = __builtin_amdgcn_mfma_i32_16x16x64_i8(A0, Bb0, cb, 0, 0, 0);
          ca = __builtin_amdgcn_mfma_i32_16x16x64_i8(A1, Ba1, ca, 0, 0, 0);
          cb = __builtin_amdgcn_mfma_i32_16x16x64_i8(A1, Bb1, cb, 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          finish_tile(tile, ca);
          finish_tile(tile + 1, cb);
        }
      };
      if constexpr (KW) {                           // the row's parameters first, then the codes
        s01[0] = *reinterpret_cast<const v2f*>(ks_row + wc0);
        m01[0] = *reinterpret_cast<const uint32_t*>(km_row + wc0);
        pin_order();
      }
#pragma unroll
      for (int d = 0; d < kRK; ++d) load_group(d, wave + d * kVisWaves);
      pin_order();
      // the lane's slice of the staged query, read while the first key groups are on their way
#pragma unroll
      for (int h = 0; h < kHeads; ++h) {
        qv0[h] = qf[h * kD + wc0] * (a.softmax_scale * variant_weight<BITS>(wvar0));
        qv1[h] = qf[h * kD + wc1] * (a.softmax_scale * variant_weight<BITS>(wvar1));
      }
      if constexpr (kPrimeValues) {
        if (a.mode != kModeExtrema) {
#pragma unroll
          for (int d = 0; d < kRingV; ++d) p2_load_tile(d, wave * 64 + d * (kVisWaves * 64));
          pin_order();
        }
      }
      if constexpr (KW) {
        build_operand(0, stage, A0w, A1w, bias_w, inv_f_w, inv_f16_w);
        pin_order();
      }
      int t = wave;
      for (; t + (kRK - 1) * kVisWaves < n_groups; t += kRK * kVisWaves) {
#pragma unroll
        for (int d = 0; d < kRK; ++d) {             // no branch around the ring's loads
          const int tt = t + d * kVisWaves;
          do_group(d, tt);
          pin_order();
          load_group(d, tt + kRK * kVisWaves);
          pin_order();
        }
      }
#pragma unroll
      for (int d = 0; d < kRK; ++d)                 // the wave's last groups, already loaded
        if (t + d * kVisWaves < n_groups) do_group(d, t + d * kVisWaves);
    }
    // fold the 16 token lanes of every head
    mn = row_min(mn);     // on the DPP network: no LDS round trips at the end of the phase
    mx = row_max(mx);
    if (n16 == 0) {
      red[(wave * kHeads + hres) * kRedPerHead + 0] = mn;
      red[(wave * kHeads + hres) * kRedPerHead + 1] = mx;
    }
  } else {
    // text logits on the fp16 matrix cores (products of fp16 numbers are exact in fp32)
    float tmax[4] = {-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX};
    if (ntx > 0) {
      v8h At[4];
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i)
          At[s][i] = n16 < gh ? (_Float16)qf[n16 * kD + 32 * s + 8 * kb + i] : (_Float16)0;
      // Loads that touch whole cache lines: a wave-wide load covers one 128-byte line of 8 tokens,
      // lanes n16 < 8 its first 64 bytes (8kb .. +7 of 32 channels), lanes n16 >= 8 the other 64.
      // Matrix columns n16 and n16 + 8 thus hold the same token with different channels: two
      // accumulators take the two matching query slices (the other half of each is discarded) and
      // the halves meet through a rotation by 8 lanes.  Twice the matrix work, which is idle
      // anyway, for half the cache-line requests.  A 16-token tile is two such 8-token halves.
      const int tsub = n16 & 7, hsel = n16 >> 3;
      // the chunk's text keys as a buffer of ntx tokens: tokens past the end (a ragged last tile, a
      // tile past the last one) read as zeros and are never stored
      const __amdgpu_buffer_rsrc_t kt_buf =
          stream_buffer(a.k_text + ((size_t)row * a.n_text_cap + txt0) * kD, (unsigned)ntx * kD * 2);
      const int kt_lane = (tsub * kD + 32 * hsel + 8 * kb) * 2;
      const int n_tiles = (ntx + 15) / 16;
      v8h kt[kRingT][4];                       // [half u][line]: index 2u + line
      auto load_tile = [&](int slot, int tile) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int tok_bytes = (tile * 16 + 8 * u) * (kD * 2);     // wave-uniform
          kt[slot][2 * u] = buffer_load_v8h<NT>(kt_buf, kt_lane, tok_bytes);           // channels 32 hsel + 8kb .. of line 0 (channels 0..63)
          kt[slot][2 * u + 1] = buffer_load_v8h<NT>(kt_buf, kt_lane + 128, tok_bytes); // the same of line 1 (channels 64..127)
        }
      };
#pragma unroll
      for (int d = 0; d < kRingT; ++d) load_tile(d, tw + d * kTextWaves);
      pin_order();
      for (int t = tw; t < n_tiles; t += kRingT * kTextWaves) {
#pragma unroll
        for (int d = 0; d < kRingT; ++d) {
          const int tile = t + d * kTextWaves;
          if (tile < n_tiles) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
              const v4f z = {0.f, 0.f, 0.f, 0.f};
              v4f cx = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[0], kt[d][2 * u], z, 0, 0, 0);
              v4f cy = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[1], kt[d][2 * u], z, 0, 0, 0);
              cx = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[2], kt[d][2 * u + 1], cx, 0, 0, 0);
              cy = __builtin_amdgcn_mfma_f32_16x16x32_f16(At[3], kt[d][2 * u + 1], cy, 0, 0, 0);
              // columns < 8 of cx and columns >= 8 of cy are the valid halves of the same tokens
              v4f c;
#pragma unroll
              for (int r = 0; r < 4; ++r) c[r] = cx[r] + dpp_f32<0x128>(cy[r]);     // row_ror 8
              const int tok = tile * 16 + 8 * u + tsub;
              // result rows 4*kb + r are heads; only heads < gh <= 4 exist, all of them in the lanes
              // with kb = 0: one test per lane, and the test per head is the same for the whole wave
              if (kb == 0 && hsel == 0 && tok < ntx) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                  if (r < gh) {
                    const float sv = c[r] * a.softmax_scale;
                    logits[r * a.stride + nv + tok] = sv;
                    tmax[r] = fmaxf(tmax[r], sv);
                  }
                }
              }
            }
          }
          pin_order();
          load_tile(d, tile + kRingT * kTextWaves);
          pin_order();
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) tmax[r] = row_max(tmax[r]);
    if (lane == 0)
      for (int r = 0; r < 4; ++r) red[(wave * kHeads + r) * kRedPerHead + 2] = tmax[r];
  }
  __syncthreads();
  if (a.mode == kModeExtrema) {
    // first pass of a split row: only the extrema of this chunk's visual logits are wanted
    if (tid < gh) {
      float lo = FLT_MAX, hi = -FLT_MAX;
      for (int w = 0; w < kVisWaves; ++w) {
        lo = fminf(lo, red[(w * kHeads + tid) * kRedPerHead + 0]);
        hi = fmaxf(hi, red[(w * kHeads + tid) * kRedPerHead + 1]);
      }
      float* mm = a.ws_minmax + ((head0 + tid) * a.n_chunks + chunk) * 2;
      mm[0] = lo;
      mm[1] = hi;
    }
    return;
  }

  // ---- phase 2 set-up: calibration line and the softmax reference point, per head.
  // Every wave folds the per-wave extrema itself, spread over its lanes: lane 16h + w reads what
  // wave w left for head h, a row reduction makes them the head's extrema.  With a split row the
  // same lanes also fold the chunk extrema of the first pass (chunk w, w + 16, ...).
  static_assert(kWaves <= 16 && kHeads == 4, "one row of 16 lanes per head");
  float lo_l = FLT_MAX, hi_l = -FLT_MAX, tm_l = -FLT_MAX, glo_l = FLT_MAX, ghi_l = -FLT_MAX;
  {
    const int h = lane >> 4, w = lane & 15;
    if (w < kVisWaves) {
      lo_l = red[(w * kHeads + h) * kRedPerHead + 0];
      hi_l = red[(w * kHeads + h) * kRedPerHead + 1];
    } else if (w < kWaves) {
      tm_l = red[(w * kHeads + h) * kRedPerHead + 2];
    }
    if (a.mode == kModePartial && a.calib_mode == CQ_CALIB_DYNAMIC && h < gh) {
      glo_l = chunk_mm[0];                  // chunk min(w, n_chunks - 1), asked for before phase 1
      ghi_l = chunk_mm[1];
      const float* mm = a.ws_minmax + (head0 + h) * a.n_chunks * 2;
      for (int cidx = w + 16; cidx < a.n_chunks; cidx += 16) {
        glo_l = fminf(glo_l, mm[2 * cidx]);
        ghi_l = fmaxf(ghi_l, mm[2 * cidx + 1]);
      }
    }
    lo_l = row_min(lo_l);
    hi_l = row_max(hi_l);
    tm_l = row_max(tm_l);
    if (a.mode == kModePartial) {
      glo_l = row_min(glo_l);
      ghi_l = row_max(ghi_l);
    }
  }
  float a2[kHeads], c2v[kHeads], c2t[kHeads], mref[kHeads];
#pragma unroll
  for (int h = 0; h < kHeads; ++h) {
    const float lo = lane_value(lo_l, 16 * h), hi = lane_value(hi_l, 16 * h);
    const float tm = lane_value(tm_l, 16 * h);
    float slope = 1.f, gam = 0.f, shift = 0.f;    // s' = slope * (s - gam) + shift
    if (a.calib_mode != CQ_CALIB_NONE && nv > 0) {
      float glo = a.gamma, ghi = a.delta;
      if (a.calib_mode == CQ_CALIB_DYNAMIC) {
        glo = lo;
        ghi = hi;
        if (a.mode == kModePartial && h < gh) {   // extrema of the whole row, from the first pass
          glo = fminf(glo, lane_value(glo_l, 16 * h));
          ghi = fmaxf(ghi, lane_value(ghi_l, 16 * h));
        }
      }
      const float width = ghi - glo;
      slope = width == 0.f ? 1.f : (width + a.tau1 - a.tau2) / width;
      gam = glo;
      shift = glo - a.tau1;
    }
    float M = tm;
    if (nv > 0) {
      M = fmaxf(M, slope * (lo - gam) + shift);
      M = fmaxf(M, slope * (hi - gam) + shift);
    }
    mref[h] = M;
    a2[h] = slope * kLog2e;
    c2v[h] = (shift - slope * gam - M) * kLog2e;
    c2t[h] = -M * kLog2e;
  }

  // =================================================================== phase 2: weighted values
  v4i acc[8];
  float facc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // banked part, already unscaled
  int Fv = 0;          // shift of this wave's accumulators at the end of phase 2
#pragma unroll
  for (int p = 0; p < 8; ++p) acc[p] = (v4i){0, 0, 0, 0};
  float lsum[kHeads] = {0.f, 0.f, 0.f, 0.f}, msum[kHeads] = {0.f, 0.f, 0.f, 0.f};
  float ttot[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // a text wave's sums, see below

  if (vis_wave) {
    if constexpr (VCH) { if (nv > 0) {
      // Channel-wise values: out_c = sum over value groups G of
      //     scale_{G,c} * sum_{j in G} p_j code_{j,c}  +  min_{G,c} * sum_{j in G} p_j.
      // The weights p_j <= 1 go into the matrix operand with one fixed shift (2^29); an extra
      // product with an all-ones operand yields sum_j p_j in the same fixed point and in the
      // accumulator layout (column = code byte, head = lane / 16).  A wave owns whole value
      // groups (v_group / 64 consecutive tiles) and folds each finished group into fp32.
      const int VG = a.v_group, tsh = VG == 128 ? 1 : 0, tpg = 1 << tsh;
      const int n_vg = nv >> (6 + tsh);      // nv / VG, VG = 64 << tsh
      const int n_my = n_vg > wave ? ((n_vg - wave + kVisWaves - 1) / kVisWaves) << tsh : 0;
      const uint32_t* vc_row = a.v_codes + ((size_t)row * a.n_vis + vis0) * (4 * BITS);
      const size_t g0 = (size_t)row * a.v_prow + (size_t)(vis0 >> (6 + tsh)) * a.v_pstride;
      // the lane's result columns are code byte n16: 8 (b = 1) or 2 x 4 (b = 2) consecutive channels
      const int c_lo = BITS == 1 ? 32 * (n16 >> 2) + 24 - 8 * (n16 & 3) : 16 * (n16 >> 2) + 12 - 4 * (n16 & 3);
      const int c_hi = BITS == 1 ? c_lo + 4 : c_lo + 64;
      const float* vsc = a.v_scale + g0;
      const uint16_t* vmn = a.v_min + g0;
      const int x_wr = ((lane >> 4) * a.stride) * 4 + (lane & 15) * 16;
      const int x_rd = (kb * a.stride) * 4 + (n16 >> 1) * 16 + (n16 & 1) * 8;
      const int v_rd = (kb * 16 + (n16 >> 1)) * (16 * BITS) + (n16 & 1) * 8;
      auto tile_start = [&](int k) {          // k-th tile of this wave, clamped to its last one
        const int kc = min(k, n_my - 1);
        return (wave + (kc >> tsh) * kVisWaves) * VG + (kc & (tpg - 1)) * 64;
      };
      v4i cg[kRingV][BITS];
      auto load_tile = [&](int slot, int k) {
        // a tile's code bytes are contiguous (64 tokens x 16b bytes): instruction e takes the e-th KB,
        // whole cache lines; the same image goes to LDS
        const int j = tile_start(k);
#pragma unroll
        for (int e = 0; e < BITS; ++e)
          cg[slot][e] = stream_load<kNtCodes>(reinterpret_cast<const v4i*>(vc_row + (size_t)j * (4 * BITS) + 256 * e + 4 * lane));
      };
      v4f gsc[2];
      v2i gmn[2];
      auto load_group = [&](int gi) {         // scales and minima of the wave's gi-th group
        const int grp = min(wave + gi * kVisWaves, n_vg - 1);
        gsc[0] = *reinterpret_cast<const v4f*>(vsc + (size_t)grp * a.v_pstride + c_lo);
        gsc[1] = *reinterpret_cast<const v4f*>(vsc + (size_t)grp * a.v_pstride + c_hi);
        gmn[0] = *reinterpret_cast<const v2i*>(vmn + (size_t)grp * a.v_pstride + c_lo);
        gmn[1] = *reinterpret_cast<const v2i*>(vmn + (size_t)grp * a.v_pstride + c_hi);
      };
      auto prep_tile = [&](int slot, int k, int buf) {
        const int jt = tile_start(k);
        float lg[kHeads];
#pragma unroll
        for (int h = 0; h < kHeads; ++h) lg[h] = logits[h * a.stride + jt + lane];
        v4i xs;
#pragma unroll
        for (int h = 0; h < kHeads; ++h) {
          const float p = __builtin_amdgcn_exp2f(fmaf(lg[h], a2[h], c2v[h]));
          lsum[h] += p;
          xs[h] = product_digits(p, 536870912.f);
        }
        __builtin_amdgcn_wave_barrier();
        *reinterpret_cast<v4i*>(lbytes + (size_t)jt * 4 + x_wr) = xs;
#pragma unroll
        for (int e = 0; e < BITS; ++e)
          *reinterpret_cast<v4i*>(stage + (BITS == 1 ? buf * 1024 : 0) + 1024 * e + 16 * lane) =
              cg[slot][e];
      };
      v4i acc_w = {0, 0, 0, 0};
      const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
      // folds the finished value group into fp32 and asks for the parameters of group `next_group`
      auto fold_group = [&](int next_group) {
        const float wsum = digits_to_float(acc_w);
        acc_w = (v4i){0, 0, 0, 0};
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          // accumulator p holds channel c_lo + 7 - p (b = 1), c_lo + 3 - p or c_hi + 3 - (p - 4)
          const int i = 7 - p;
          const int vec = BITS == 1 ? i >> 2 : p >> 2, el = BITS == 1 ? i & 3 : 3 - (p & 3);
          const uint32_t mpair = (uint32_t)gmn[vec][el >> 1];
          const float mn = __half2float(__ushort_as_half((uint16_t)((el & 1) ? mpair >> 16 : mpair & 0xffffu)));
          // the operand byte of a set code is 2^p (b = 1) resp. code * {1, 4, 16, 16}: take that out
          const float sc = gsc[vec][el] * variant_weight<BITS>(p % (8 / BITS));
          facc[p] = fmaf(digits_to_float(acc[p]), sc, fmaf(wsum, mn, facc[p]));
          acc[p] = (v4i){0, 0, 0, 0};
        }
        pin_order();
        load_group(next_group);
        pin_order();
      };
      // FOLD: the tile ends a value group, whose sums are folded into fp32 and whose successor's
      // parameters are asked for.  It is a compile-time property of the call site, so that every
      // step issues the same loads whatever happens at run time: with a branch around loads the
      // compiler drained all outstanding loads in every step (`s_waitcnt vmcnt(0)`), which took the
      // ring of value tiles out of flight.
      auto m_step = [&](int k, int d, auto fold_tag) {
        constexpr bool FOLD = decltype(fold_tag)::value;
        const int buf = d & 1;
        const int jt = tile_start(k);
        const uint8_t* xr = lbytes + (size_t)jt * 4 + x_rd;
        const uint8_t* vr = stage + (BITS == 1 ? buf * 1024 : 0) + v_rd;
        const v2i a_lo = lds_read_tr8(xr), a_hi = lds_read_tr8(xr + 128);
        const v4i A = {a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
        v4i raw[BITS];
#pragma unroll
        for (int cb = 0; cb < BITS; ++cb) {
          const v2i b_lo = lds_read_tr8(vr + 16 * cb), b_hi = lds_read_tr8(vr + 16 * cb + 128 * BITS);
          raw[cb] = (v4i){b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
        }
        const int nslot = (d + 1) % kRingV;
        if (k + 1 < n_my) prep_tile(nslot, k + 1, buf ^ 1);
        pin_order();
        load_tile(nslot, k + 1 + kRingV);
        pin_order();
        auto variant_of = [&](int p) {
          v4i B;
#pragma unroll
          for (int v = 0; v < 4; ++v)
            B[v] = operand_variant<BITS>((uint32_t)raw[p / (8 / BITS)][v], p % (8 / BITS));
          return B;
        };
        v4i Bn = variant_of(0);
#pragma unroll
        for (int p = 0; p < 8; ++p) {       // operand p + 1 is formed before product p is issued
          const v4i B = Bn;
          if (p < 7) Bn = variant_of(p + 1);
          __builtin_amdgcn_sched_barrier(0);
          acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, B, acc[p], 0, 0, 0);
        }
        acc_w = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, ones, acc_w, 0, 0, 0);
        if constexpr (FOLD) fold_group((k >> tsh) + 1);
        lds_publish();
      };
      if (n_my > 0) {
#pragma unroll
        for (int d = 0; d < kRingV; ++d) load_tile(d, d);
        load_group(0);
        prep_tile(0, 0, 0);
        lds_publish();
        load_tile(0, kRingV);
        pin_order();
        static_assert(kRingV == 2, "the loops below pair a ring slot with a tile of a 128-token group");
        const std::integral_constant<bool, true> fold_yes;
        const std::integral_constant<bool, false> fold_no;
        if (a.v_pstride == 0) {
          // whole-sequence statistics: every group has the row's parameters, so the wave folds
          // once, after its last tile (an int32 accumulator takes 2^20 per tile at most: 2047
          // tiles, a workgroup's LDS holds ~140)
          int k = 0;
          for (; k + 2 <= n_my; k += 2) {
            m_step(k, 0, fold_no);
            m_step(k + 1, 1, fold_no);
          }
          if (k < n_my) m_step(k, 0, fold_no);
          fold_group(0);
        } else if (tpg == 2) {              // groups of 128 tokens: two tiles, the second one folds
          for (int k = 0; k < n_my; k += 2) {
            m_step(k, 0, fold_no);
            m_step(k + 1, 1, fold_yes);
          }
        } else {                            // groups of 64 tokens: every tile folds
          int k = 0;
          for (; k + 2 <= n_my; k += 2) {
            m_step(k, 0, fold_yes);
            m_step(k + 1, 1, fold_yes);
          }
          if (k < n_my) m_step(k, 0, fold_yes);
        }
      }
      Fv = 0;
    } }
    if constexpr (!VCH && BITS > 2) { if (nv > 0) {
      // 4- and 8-bit codes: a tile's code bytes (64 or 128 per token) go through the wave's 2 KB
      // staging buffer two column blocks at a time, straight from the ring registers; the steps
      // of a tile run one after the other (these widths are bound by their bytes, not by issue).
      constexpr int kV = 8 / BITS;
      int F_prep = 90, F_acc = 90;
      float fit_below = ldexpf(1.f, 29 - 90);
      const uint32_t* vc_row = a.v_codes + ((size_t)row * a.n_vis + vis0) * (4 * BITS);
      const int step = kVisWaves * 64, last = nv - 64;
      const int x_wr = ((lane >> 4) * a.stride) * 4 + (lane & 15) * 16;
      const int x_rd = (kb * a.stride) * 4 + (n16 >> 1) * 16 + (n16 & 1) * 8;
      const int v_rd = (kb * 16 + (n16 >> 1)) * 32 + (n16 & 1) * 8;     // 32-byte rows: two blocks
      v4i cg[2][BITS];
      float vsr[2];
      uint16_t vmr[2];
      auto load_tile = [&](int slot, int jt) {
        const int j = min(jt, last) + lane;
#pragma unroll
        for (int e = 0; e < BITS; ++e)
          cg[slot][e] = stream_load<kNtCodes>(reinterpret_cast<const v4i*>(vc_row + (size_t)j * (4 * BITS) + 4 * e));
        vsr[slot] = stream_load<NT>(vs_row + j);
        vmr[slot] = stream_load<NT>(vm_row + j);
      };
      auto tile_step = [&](int jt, int slot) {
        if (__builtin_amdgcn_ballot_w64(vsr[slot] >= fit_below) != 0) {
          F_prep = min(F_prep, fixed_point_shift(wave_max_nonneg(vsr[slot])));
          fit_below = ldexpf(1.f, 29 - F_prep);
        }
        if (F_prep < F_acc) {                     // bank before a tile with a lower shift is added
          const float w_old = ldexpf(1.f, -F_acc);
#pragma unroll
          for (int p = 0; p < 8; ++p) {
            facc[p] = fmaf(digits_to_float(acc[p]), w_old, facc[p]);
            acc[p] = (v4i){0, 0, 0, 0};
          }
          F_acc = F_prep;
        }
        const float vsf = ldexpf(vsr[slot], F_prep);
        // 8-bit operands are code - 128: the 128 comes back with the token's minimum
        const float vmf = __half2float(__ushort_as_half(vmr[slot])) + (BITS == 8 ? 128.f * vsr[slot] : 0.f);
        v4i xs;
#pragma unroll
        for (int h = 0; h < kHeads; ++h) {
          const float p = __builtin_amdgcn_exp2f(fmaf(logits[h * a.stride + jt + lane], a2[h], c2v[h]));
          lsum[h] += p;
          msum[h] = fmaf(p, vmf, msum[h]);
          xs[h] = product_digits(p, vsf);
        }
        __builtin_amdgcn_wave_barrier();
        *reinterpret_cast<v4i*>(lbytes + (size_t)jt * 4 + x_wr) = xs;
        lds_publish();
        const uint8_t* xr = lbytes + (size_t)jt * 4 + x_rd;
        const v2i a_lo = lds_read_tr8(xr), a_hi = lds_read_tr8(xr + 128);
        const v4i A = {a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
#pragma unroll
        for (int r = 0; r < BITS / 2; ++r) {
          __builtin_amdgcn_wave_barrier();
          *reinterpret_cast<v4i*>(stage + lane * 32) = cg[slot][2 * r];
          *reinterpret_cast<v4i*>(stage + lane * 32 + 16) = cg[slot][2 * r + 1];
          lds_publish();
#pragma unroll
          for (int cbl = 0; cbl < 2; ++cbl) {
            const v2i b_lo = lds_read_tr8(stage + v_rd + 16 * cbl);
            const v2i b_hi = lds_read_tr8(stage + v_rd + 16 * cbl + 256);
            const v4i raw = {b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
#pragma unroll
            for (int v = 0; v < kV; ++v) {
              v4i B;
#pragma unroll
              for (int u = 0; u < 4; ++u) B[u] = operand_variant<BITS>((uint32_t)raw[u], v);
              const int p = (2 * r + cbl) * kV + v;
              acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, B, acc[p], 0, 0, 0);
            }
          }
        }
        pin_order();
        load_tile(slot, jt + 2 * step);
        pin_order();
      };
      const int j_first = wave * 64;
      load_tile(0, j_first);
      load_tile(1, j_first + step);
      pin_order();
      int j0 = j_first;
      for (; j0 + step < nv; j0 += 2 * step) {        // no branch around the ring's loads in here
        tile_step(j0, 0);
        tile_step(j0 + step, 1);
      }
      if (j0 < nv) tile_step(j0, 0);
      Fv = F_acc;
    } }
    if constexpr (!VCH && BITS <= 2) { if (nv > 0) {
      // Pipeline over 64-token tiles (tile k of this wave starts at token (wave + 8k) * 64):
      //   G(k)  global loads of the tile's codes, scale and min into a ring of registers
      //   P(k)  weights p = 2^(a2*s + c2) from the logits in LDS, their fixed-point digits X(k)
      //         and the raw code bytes back to LDS
      //   M(k)  transposing reads of X(k) and the codes, 8 x (4 AND + 1 MFMA)
      // One step runs M(k), P(k+1) and G(k+1+kRingV); M(k) and P(k+1) are independent, so the
      // matrix pipe and the VALU overlap.  X(k) overwrites the tile's own logits (1 KB for
      // 4 heads x 64 tokens, dead once read); the code bytes alternate between two buffers.
      // running fixed-point shift: set by the largest value scale met so far; when a tile lowers
      // it, the integer accumulators are banked into fp32 before that tile is added
      int F_prep = 90, F_acc = 90, F_tile[2] = {90, 90};
      float fit_below = ldexpf(1.f, 29 - 90);   // scales below this fit the shift F_prep
      const int step = kVisWaves * 64;
      const int x_wr = ((lane >> 4) * a.stride) * 4 + (lane & 15) * 16;          // row of token lane
      const int x_rd = (kb * a.stride) * 4 + (n16 >> 1) * 16 + (n16 & 1) * 8;   // tr rows 16kb+k
      const int v_rd = (kb * 16 + (n16 >> 1)) * (16 * BITS) + (n16 & 1) * 8;
      auto& cg = p2_cg;
      auto& vsr = p2_vsr;
      auto& vmr = p2_vmr;
      auto& load_tile = p2_load_tile;
      auto prep_tile = [&](int slot, int jt, int buf) {
        if (__builtin_amdgcn_ballot_w64(vsr[slot] >= fit_below) != 0) {
          // some token's scale does not fit the running shift (rare after the first tiles)
          F_prep = min(F_prep, fixed_point_shift(wave_max_nonneg(vsr[slot])));
          fit_below = ldexpf(1.f, 29 - F_prep);
        }
        F_tile[buf] = F_prep;
        const float vsf = ldexpf(vsr[slot], F_prep);
        // converted here and now: folded into the multiply-adds below, the raw 16 bits would stay
        // live past the ring's next load into this slot, the compiler would give that load another
        // register and copy it back at the loop's end - behind a wait for every outstanding load
        float vmf = __half2float(__ushort_as_half(vmr[slot]));
        asm volatile("" : "+v"(vmf));
        float lg[kHeads];
#pragma unroll
        for (int h = 0; h < kHeads; ++h) lg[h] = logits[h * a.stride + jt + lane];
        v4i xs;
#pragma unroll
        for (int h = 0; h < kHeads; ++h) {
          const float p = __builtin_amdgcn_exp2f(fmaf(lg[h], a2[h], c2v[h]));
          lsum[h] += p;
          msum[h] = fmaf(p, vmf, msum[h]);
          xs[h] = product_digits(p, vsf);
        }
        __builtin_amdgcn_wave_barrier();
        *reinterpret_cast<v4i*>(lbytes + (size_t)jt * 4 + x_wr) = xs;
        // b = 1: two 1 KB buffers alternate; b = 2: one 2 KB buffer (LDS executes a wave's
        // accesses in order, so the previous tile's reads are served before these writes)
#pragma unroll
        for (int e = 0; e < BITS; ++e)
          *reinterpret_cast<v4i*>(stage + (BITS == 1 ? buf * 1024 : 0) + 1024 * e + 16 * lane) =
              cg[slot][e];
      };
      const int j_first = wave * 64;      // the ring's first tiles were asked for in phase 1
      if (j_first < nv) {
        prep_tile(0, j_first, 0);
        lds_publish();
      }
      load_tile(0, j_first + kRingV * step);
      pin_order();
      // one step: M(tile jt) with P(next tile) and G(next tile + kRingV) in its shadow.  In the
      // main loop every step has a next tile, so the body is free of branches around the ring's
      // loads (the compiler then counts outstanding loads exactly instead of draining them).
      auto m_step = [&](int jt, int d, bool always_prep) {
        const int buf = d & 1;
        const uint8_t* xr = lbytes + (size_t)jt * 4 + x_rd;
        const uint8_t* vr = stage + (BITS == 1 ? buf * 1024 : 0) + v_rd;
        const v2i a_lo = lds_read_tr8(xr), a_hi = lds_read_tr8(xr + 128);
        const v4i A = {a_lo[0], a_lo[1], a_hi[0], a_hi[1]};
        // code bytes: column block cb covers bytes 16cb .. 16cb+15 of every token
        v4i raw[BITS];
#pragma unroll
        for (int cb = 0; cb < BITS; ++cb) {
          const v2i b_lo = lds_read_tr8(vr + 16 * cb), b_hi = lds_read_tr8(vr + 16 * cb + 128 * BITS);
          raw[cb] = (v4i){b_lo[0], b_lo[1], b_hi[0], b_hi[1]};
        }
        const int nslot = (d + 1) % kRingV;
        if (always_prep || jt + step < nv) prep_tile(nslot, jt + step, buf ^ 1);
        pin_order();
        load_tile(nslot, jt + step + kRingV * step);
        pin_order();
        if (F_tile[buf] < F_acc) {              // wave-uniform, rare
          // a larger scale lowered the shift: bank what was accumulated so far in fp32 (the
          // four digit accumulators of a value cannot be shifted independently)
          const float w_old = ldexpf(1.f, -F_acc);
#pragma unroll
          for (int p = 0; p < 8; ++p) {
            facc[p] = fmaf(digits_to_float(acc[p]), w_old, facc[p]);
            acc[p] = (v4i){0, 0, 0, 0};
          }
          F_acc = F_tile[buf];
        }
        // p = mask variant (b = 1) or 4 * block + variant; the operand of product p + 1 is formed
        // before product p is issued, so no product waits on the ANDs right in front of it
        auto variant_of = [&](int p) {
          v4i B;
#pragma unroll
          for (int v = 0; v < 4; ++v)
            B[v] = operand_variant<BITS>((uint32_t)raw[p / (8 / BITS)][v], p % (8 / BITS));
          return B;
        };
        v4i Bn = variant_of(0);
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const v4i B = Bn;
          if (p < 7) Bn = variant_of(p + 1);
          __builtin_amdgcn_sched_barrier(0);
          acc[p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, B, acc[p], 0, 0, 0);
        }
        lds_publish();
      };
      int j0 = j_first;
      for (; j0 + kRingV * step < nv; j0 += kRingV * step) {     // all kRingV next tiles exist
#pragma unroll
        for (int d = 0; d < kRingV; ++d) m_step(j0 + d * step, d, true);
      }
#pragma unroll
      for (int d = 0; d < kRingV; ++d)                            // the wave's last 1..kRingV tiles
        if (j0 + d * step < nv) m_step(j0 + d * step, d, false);
      Fv = F_acc;
    } }
  } else {
    // text tail.  lane = (token slot kb, channels 8 * n16 .. +7): one 16-byte load covers 8 channels
    // of one token, a wave-wide load covers 4 tokens.  The contraction over tokens runs on the
    // matrix cores as 16 independent 4 x 4 x 4 products per instruction (heads x channels x
    // tokens; fp16 operands, fp32 sums): a 4 x 4 transpose over the wave's four rows of lanes
    // (two lane swaps each way) and four byte permutes leave every lane with the four tokens of
    // its two channels 8 n16 + 2 kb, + 1, and the weights come as fp16 pairs hi + lo / 2^11 of
    // 2^10 p (p <= 1; products of fp16 numbers are exact in fp32), so the sum carries the weights
    // to 2^-22 as the fp32 multiply-adds it replaces did to 2^-24.  The tail is handed to the text
    // waves in shares of SH tokens; the weights of a share are computed once (lane = token) and
    // staged in the share's own logit slots (SH * 4 bytes in each of the four head rows), one
    // 64-byte record per load step: [hi | lo][head][token of the step].
    // Shares of 64 tokens are the efficient ones; a short tail (a split row's chunk, a small
    // prompt) goes out in shares of 16 so that it still occupies all text waves.
    float tl[kHeads] = {0.f, 0.f, 0.f, 0.f};
    if (ntx > 0) {
      // the chunk's text values as a buffer of ntx tokens (reads past the end return zeros, which
      // meet weights of zero)
      const __amdgpu_buffer_rsrc_t vt_buf =
          stream_buffer(a.v_text + ((size_t)row * a.n_text_cap + txt0) * kD, (unsigned)ntx * kD * 2);
      const int vt_lane = (kb * kD + 8 * n16) * 2;
      v4f acc_hi[2], acc_lo[2];              // [channel 8 n16 + 2 kb + i][head]
#pragma unroll
      for (int i = 0; i < 2; ++i) acc_hi[i] = acc_lo[i] = (v4f){0.f, 0.f, 0.f, 0.f};
      auto text_values = [&](auto share_tag) {
        constexpr int SH = decltype(share_tag)::value;
        // wave-wide loads per share, how many of them are in flight, records per head row
        constexpr int kSteps = SH / 4, kDepth = kRingTV < kSteps ? kRingTV : kSteps, kRecs = SH / 16;
        static_assert(kSteps % kDepth == 0, "the ring divides a share");
        const int n_sh = (ntx + SH - 1) / SH;
        const int rec_wr = (((lane >> 2) / kRecs) * a.stride) * 4 + ((lane >> 2) % kRecs) * 64 + (lane & 3) * 2;
        const int rec_rd = (lane & 3) * 8;          // matrix row = lane % 4 = head
        v8h ring[kDepth];
        auto load_step = [&](int slot, int sh, int s) {
          ring[slot] = buffer_load_v8h<NT>(vt_buf, vt_lane, (sh * SH + 4 * s) * (kD * 2));
        };
#pragma unroll
        for (int s = 0; s < kDepth; ++s) load_step(s, tw, s);
        pin_order();
        for (int sh = tw; sh < n_sh; sh += kTextWaves) {
          const int t0 = sh * SH;
          const int nt = min(SH, ntx - t0);
          v4f pv = {0.f, 0.f, 0.f, 0.f};
          if (lane < nt) {
#pragma unroll
            for (int h = 0; h < kHeads; ++h)
              if (h < gh)
                pv[h] = __builtin_amdgcn_exp2f(
                    fmaf(logits[h * a.stride + nv + t0 + lane], kLog2e, c2t[h]));
          }
#pragma unroll
          for (int h = 0; h < kHeads; ++h) tl[h] += pv[h];
          uint8_t* pb = lbytes + (size_t)(nv + t0) * 4;
          __builtin_amdgcn_wave_barrier();
          asm volatile("" ::: "memory");     // the records overwrite logits read just above
          if (lane < SH) {                                                  // zero beyond nt
#pragma unroll
            for (int h = 0; h < kHeads; ++h) {
              const float ps = pv[h] * 1024.f;
              const _Float16 hi = (_Float16)ps;
              const _Float16 lo = (_Float16)((ps - (float)hi) * 2048.f);
              *reinterpret_cast<_Float16*>(pb + rec_wr + 8 * h) = hi;
              *reinterpret_cast<_Float16*>(pb + rec_wr + 32 + 8 * h) = lo;
            }
          }
          lds_publish();
#pragma unroll
          for (int s = 0; s < kSteps; ++s) {
            const int slot = s % kDepth;
            const uint8_t* rec = pb + ((s / kRecs) * a.stride) * 4 + (s % kRecs) * 64 + rec_rd;
            const v4h p_hi = *reinterpret_cast<const v4h*>(rec);
            const v4h p_lo = *reinterpret_cast<const v4h*>(rec + 32);
            const v4u32 raw = __builtin_bit_cast(v4u32, ring[slot]);
            // word j of token kb -> row j of lanes holds word j of tokens 0..3
            const v2u lo2 = __builtin_amdgcn_permlane32_swap(raw[0], raw[2], false, false);
            const v2u hi2 = __builtin_amdgcn_permlane32_swap(raw[1], raw[3], false, false);
            const v2u t01 = __builtin_amdgcn_permlane16_swap(lo2[0], hi2[0], false, false);
            const v2u t23 = __builtin_amdgcn_permlane16_swap(lo2[1], hi2[1], false, false);
            // the even channel's four tokens from the low halves, the odd channel's from the high
            const v2u even = {__builtin_amdgcn_perm(t01[1], t01[0], 0x05040100u),
                              __builtin_amdgcn_perm(t23[1], t23[0], 0x05040100u)};
            const v2u odd = {__builtin_amdgcn_perm(t01[1], t01[0], 0x07060302u),
                             __builtin_amdgcn_perm(t23[1], t23[0], 0x07060302u)};
            const v4h v_even = __builtin_bit_cast(v4h, even), v_odd = __builtin_bit_cast(v4h, odd);
            acc_hi[0] = __builtin_amdgcn_mfma_f32_4x4x4f16(p_hi, v_even, acc_hi[0], 0, 0, 0);
            acc_hi[1] = __builtin_amdgcn_mfma_f32_4x4x4f16(p_hi, v_odd, acc_hi[1], 0, 0, 0);
            acc_lo[0] = __builtin_amdgcn_mfma_f32_4x4x4f16(p_lo, v_even, acc_lo[0], 0, 0, 0);
            acc_lo[1] = __builtin_amdgcn_mfma_f32_4x4x4f16(p_lo, v_odd, acc_lo[1], 0, 0, 0);
            // refill: step s + kDepth of this share, or the start of the wave's next share
            if (s + kDepth < kSteps) load_step(slot, sh, s + kDepth);
            else load_step(slot, sh + kTextWaves, s + kDepth - kSteps);
            pin_order();
          }
        }
      };
      // rounds of shares over the text waves, a share of 16 costing ~1.1 quarters of one of 64
      const int rounds64 = ((ntx + 63) / 64 + kTextWaves - 1) / kTextWaves;
      const int rounds16 = ((ntx + 15) / 16 + kTextWaves - 1) / kTextWaves;
      if (11 * rounds16 < 40 * rounds64) text_values(std::integral_constant<int, 16>{});
      else text_values(std::integral_constant<int, 64>{});
      // lane (kb, n16): the wave's sums for heads 0..3, channels 8 n16 + 2 kb and + 1
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int h = 0; h < kHeads; ++h)
          ttot[2 * h + i] = fmaf(acc_lo[i][h], 0x1p-11f, acc_hi[i][h]) * 0x1p-10f;
    }
#pragma unroll
    for (int h = 0; h < kHeads; ++h) lsum[h] = tl[h];
  }
  __syncthreads();    // logits are dead from here on; their LDS becomes the partial buffer

  float* partial = reinterpret_cast<float*>(smem) + (size_t)wave * kHeads * kD;   // [head][channel]
  if (vis_wave) {
    // matrix result lane: column n16 = code byte index, head = kb; accumulator p = bit position
    const float inv_fv = ldexpf(1.f, -Fv);
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const float v = fmaf(digits_to_float(acc[p]), inv_fv, facc[p]);
      // accumulator p = (column block cb, variant v) = (p / (8/b), p % (8/b)); its column n16 is byte
      // 16 cb + n16 of the token's code bytes
      constexpr int kV = 8 / BITS;
      const int tb = 16 * (p / kV) + n16;
      const int ch = (32 / BITS) * (tb >> 2) + code_in_word<BITS>(tb & 3, p % kV);
      // channel-wise values are accumulated in units of 2^-29 (the weights' fixed point)
      partial[kb * kD + ch] = VCH ? v * 0x1p-29f : v * variant_weight<BITS>(p % kV);
    }
  } else {      // text wave: lane (kb, n16) holds heads 0..3, channels 8 n16 + 2 kb and + 1
#pragma unroll
    for (int h = 0; h < kHeads; ++h)
      *reinterpret_cast<v2f*>(partial + h * kD + 8 * n16 + 2 * kb) = (v2f){ttot[2 * h], ttot[2 * h + 1]};
  }
  // The per-wave sums of the weights (l) and of the additive value term (m), four heads each: a
  // transposing fold over the wave's rows of lanes with paired swaps (a swap of two values and one
  // add halve both), then one row reduction per register: rows 0..3 of the first register end up
  // with l[0], l[1], m[0], m[1], those of the second with l[2], l[3], m[2], m[3].
  {
    auto bits_of = [](float v) { return __builtin_bit_cast(unsigned, v); };
    auto float_of = [](unsigned v) { return __builtin_bit_cast(float, v); };
    float lm[kHeads];                       // l of head h in lanes 0-31, m of head h in lanes 32-63
#pragma unroll
    for (int h = 0; h < kHeads; ++h) {
      const auto r = __builtin_amdgcn_permlane32_swap(bits_of(lsum[h]), bits_of(msum[h]), false, false);
      lm[h] = float_of(r[0]) + float_of(r[1]);
    }
#pragma unroll
    for (int pair = 0; pair < 2; ++pair) {
      const auto r = __builtin_amdgcn_permlane16_swap(bits_of(lm[2 * pair]), bits_of(lm[2 * pair + 1]), false, false);
      const float tot = row_sum(float_of(r[0]) + float_of(r[1]));
      if (n16 == 0)     // row kb: head 2 pair + (kb & 1), l for kb < 2 and m for kb >= 2
        red[(wave * kHeads + 2 * pair + (kb & 1)) * kRedPerHead + 3 + (kb >> 1)] = tot;
    }
    if (wave == 0 && lane == 0) {
#pragma unroll
      for (int h = 0; h < kHeads; ++h) red[h * kRedPerHead + 5] = mref[h];
    }
  }
  __syncthreads();

  // ---- epilogue: sum the waves, add the additive value term, normalise, round to fp16
  if (tid < kHeads * kD) {
    const int h = tid / kD, c = tid % kD;
    if (h < gh) {
      // the per-wave sums of the weights and of the additive value term: lane w of each row of 16
      // lanes fetches wave w's, a row reduction adds them (a wave works on one head: 128 = 2 x 64)
      const int wl = lane & 15;
      float l = wl < kWaves ? red[(wl * kHeads + h) * kRedPerHead + 3] : 0.f;
      float m = wl < kWaves ? red[(wl * kHeads + h) * kRedPerHead + 4] : 0.f;
      l = row_sum(l);
      m = row_sum(m);
      float num = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w)
        num += reinterpret_cast<float*>(smem)[((size_t)w * kHeads + h) * kD + c];
      if (a.mode == kModeFull) {
        a.out[(head0 + h) * kD + c] = __float2half_rn((num + m) / l);
      } else {          // one (m, l, acc[d]) partial of the joint softmax per (head, chunk)
        float* part = a.ws_partial + ((head0 + h) * a.n_chunks + chunk) * (size_t)(kD + 2);
        if (c == 0) { part[0] = red[h * kRedPerHead + 5]; part[1] = l; }
        part[2 + c] = num + m;
      }
    }
  }
}

}  // namespace


size_t fused_lds_bytes(int n_vis_chunk, int n_text_chunk, int k_group, int* stride_out) {
  // text slots are rounded up to whole 64-token blocks (a block's weights are staged in place)
  int stride = n_vis_chunk + (n_text_chunk + 63) / 64 * 64;
  stride += (16 - (stride % 32) + 32) % 32;      // stride = 16 (mod 32): conflict-free head rows
  if (stride_out) *stride_out = stride;
  size_t off = (size_t)kHeads * stride * sizeof(float);
  const size_t part = (size_t)kWaves * kHeads * kD * sizeof(float);
  if (off < part) off = part;
  off += kHeads * kD * sizeof(float);
  (void)k_group;
  off = (off + 15) & ~(size_t)15;
  off += (size_t)kVisWaves * kStageBytes;
  off += (size_t)kWaves * kHeads * kRedPerHead * sizeof(float);
  return off;
}

namespace {

constexpr int kMaxDevices = 64;

// Compute units of the current device (cached per device; 256, the MI355X count, when there is
// no device, as in host-only checks of the plan).
long long device_cu_count() {
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

// Channel-wise statistics over the whole sequence (group = n_vis, the scheme of Sec. 3.1 as
// printed) run as processing groups of 128 tokens that share the row's one parameter group.
// Returns the shape the kernel works on.
DecodeShape processing_shape(const DecodeShape& s, bool* k_whole, bool* v_whole) {
  DecodeShape e = s;
  *k_whole = s.k_axis == CQ_AXIS_CHANNEL && s.k_group == s.n_vis && s.n_vis > 128 && s.n_vis % 128 == 0;
  *v_whole = s.v_axis == CQ_AXIS_CHANNEL && s.v_group == s.n_vis && s.n_vis > 128 && s.n_vis % 128 == 0;
  if (*k_whole) e.k_group = 128;
  if (*v_whole) e.v_group = 128;
  return e;
}

// Chunks of a split row start at multiples of `unit` key groups: whole 64-token value tiles and,
// with channel-wise values, whole value groups.
int chunk_unit(const DecodeShape& s) {
  int align = 64;
  if (s.v_axis == CQ_AXIS_CHANNEL && s.v_group > align) align = s.v_group;
  return align / s.k_group > 1 ? align / s.k_group : 1;
}

// largest chunk of a row split into n_chunks (same arithmetic as the kernel)
void chunk_extent(const DecodeShape& s, int n_chunks, int* nv_max, int* nt_max) {
  const int unit = chunk_unit(s);
  const int n_units = s.n_vis / (s.k_group * unit);
  const int n_tblocks = (s.n_text + 63) / 64;
  *nv_max = 0;
  *nt_max = 0;
  for (int c = 0; c < n_chunks; ++c) {
    const int ga = chunk_first(n_units / n_chunks, n_units % n_chunks, c) * unit;
    const int gb = chunk_first(n_units / n_chunks, n_units % n_chunks, c + 1) * unit;
    const int ba = chunk_first(n_tblocks / n_chunks, n_tblocks % n_chunks, c);
    const int bb = chunk_first(n_tblocks / n_chunks, n_tblocks % n_chunks, c + 1);
    const int nv = (gb - ga) * s.k_group;
    int nt = (bb * 64 < s.n_text ? bb * 64 : s.n_text) - ba * 64;
    if (nt < 0) nt = 0;
    if (nv > *nv_max) *nv_max = nv;
    if (nt > *nt_max) *nt_max = nt;
  }
}

}  // namespace

FusedPlan make_fused_plan(const DecodeShape& shape, int min_chunks) {
  FusedPlan p;
  bool k_whole, v_whole;
  const DecodeShape s = processing_shape(shape, &k_whole, &v_whole);
  if (s.d != kD || (s.bits != 1 && s.bits != 2 && s.bits != 4 && s.bits != 8)) return p;
  if (s.bits > 2 && s.v_axis != CQ_AXIS_TOKEN) return p;     // wide codes: token-wise values only
  if (s.k_axis != CQ_AXIS_CHANNEL) return p;
  if (s.v_axis == CQ_AXIS_TOKEN ? s.v_group != kD : (s.v_group != 64 && s.v_group != 128)) return p;
  if (s.k_group != 32 && s.k_group != 64 && s.k_group != 128) return p;
  if (s.g > 2 * kHeads || s.n_vis % 64 != 0) return p;
  if (s.v_axis == CQ_AXIS_CHANNEL && s.n_vis % s.v_group != 0) return p;
  p.nhb = (s.g + kHeads - 1) / kHeads;
  const long long rows = (long long)s.B * s.Hkv * p.nhb;
  const int unit = chunk_unit(s);
  const int n_units = s.n_vis / (s.k_group * unit);
  const int max_chunks = n_units < 64 ? (n_units > 0 ? n_units : 1) : 64;
  // Fewest chunks that fit LDS.  Splitting a row that fits only to fill idle CUs does not pay:
  // every chunk repeats the fixed per-workgroup work and the logits are computed twice
  // (measured on the 128-row configuration: 24 us whole rows, 35 us in 2 chunks, 57 us in 4).
  int want = min_chunks >= 1 ? min_chunks : 1;                 // > 1: a test's or a tuner's override
  if (want > max_chunks) want = max_chunks;
  const bool forced = want > 1;
  for (int c = want; c <= max_chunks; ++c) {
    int nv, nt, stride;
    chunk_extent(s, c, &nv, &nt);
    const size_t lds = fused_lds_bytes(nv, nt, s.k_group, &stride);
    if (lds <= 160 * 1024) {
      p.n_chunks = c;
      p.stride = stride;
      p.lds = lds;
      break;
    }
  }
  if (p.lds == 0) return p;
  if (p.n_chunks > 1 && !forced) {
    // A row that has to be split anyway: a few more chunks can fill the last round of
    // workgroups.  Cost of c chunks ~ rounds over the CUs x (tokens per chunk + a fixed cost per
    // workgroup worth ~1500 tokens).
    const long long cus = device_cu_count();
    long long best_cost = -1;
    int best_c = p.n_chunks;
    const int c_hi = 3 * p.n_chunks < max_chunks ? 3 * p.n_chunks : max_chunks;
    for (int c = p.n_chunks; c <= c_hi; ++c) {
      int nv, nt;
      chunk_extent(s, c, &nv, &nt);
      const long long rounds = (rows * c + cus - 1) / cus;
      const long long cost = rounds * (nv + nt + 1500);
      if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_c = c; }
    }
    if (best_c != p.n_chunks) {
      int nv, nt, stride;
      chunk_extent(s, best_c, &nv, &nt);
      p.n_chunks = best_c;
      p.lds = fused_lds_bytes(nv, nt, s.k_group, &stride);
      p.stride = stride;
    }
  }
  if (p.n_chunks > 1 || p.nhb > 1) {
    if (s.n_vis == 0) return p;
    const size_t heads = (size_t)s.B * s.Hq;
    // chunk extrema of the visual logits (read only with dynamic calibration; 12 KB on the
    // long-context configuration), then one (m, l, acc[d]) partial per (head, chunk)
    p.ws_minmax_floats = (heads * p.n_chunks * 2 + 63) / 64 * 64;
    const size_t floats = p.ws_minmax_floats + heads * p.n_chunks * (size_t)(kD + 2);
    p.ws_bytes = (floats * sizeof(float) + 255) / 256 * 256;
  }
  p.ok = true;
  return p;
}

hipError_t launch_decode_fused(const DecodeShape& shape, const FusedPlan& plan, const void* q,
                               const cq_qtensor_t& k, const cq_qtensor_t& v, const void* k_text,
                               const void* v_text, const int32_t* n_text_dev, const Calib& calib,
                               float softmax_scale, void* out, float* workspace,
                               hipStream_t stream) {
  if (!plan.ok) return hipErrorInvalidValue;
  bool k_whole, v_whole;
  const DecodeShape s = processing_shape(shape, &k_whole, &v_whole);
  FusedArgs a;
  a.q = static_cast<const __half*>(q);
  a.k_codes = k.codes; a.k_scale = k.scale; a.k_min = k.min;
  a.v_codes = v.codes; a.v_scale = v.scale; a.v_min = v.min;
  a.k_text = static_cast<const __half*>(k_text);
  a.v_text = static_cast<const __half*>(v_text);
  a.out = static_cast<__half*>(out);
  a.Hq = s.Hq; a.Hkv = s.Hkv; a.g = s.g; a.n_vis = s.n_vis; a.n_text = s.n_text;
  a.n_text_cap = s.n_text_cap; a.n_text_dev = n_text_dev; a.k_group = s.k_group;
  a.v_group = s.v_group; a.unit = chunk_unit(s);
  a.k_prow = k_whole ? kD : s.n_vis / s.k_group * kD;
  a.k_pstride = k_whole ? 0 : kD;
  a.v_prow = a.v_pstride = 0;
  if (s.v_axis == CQ_AXIS_CHANNEL) {
    a.v_prow = v_whole ? kD : s.n_vis / s.v_group * kD;
    a.v_pstride = v_whole ? 0 : kD;
  }
  a.calib_mode = calib.mode; a.tau1 = calib.tau1; a.tau2 = calib.tau2;
  a.gamma = calib.gamma; a.delta = calib.delta; a.softmax_scale = softmax_scale;
  a.stride = plan.stride;
  a.n_chunks = plan.n_chunks;
  a.nhb = plan.nhb;
  a.ws_minmax = workspace;
  a.ws_partial = workspace ? workspace + plan.ws_minmax_floats : nullptr;
  void (*kern)(const FusedArgs) = nullptr;
  int slot = 0;
  const bool vch = s.v_axis == CQ_AXIS_CHANNEL;
  if (k_whole) {
    switch (s.bits * 2 + (vch ? 1 : 0)) {
      case 1 * 2: kern = fused_row_kernel<8, 1, false, true>; slot = 18; break;
      case 2 * 2: kern = fused_row_kernel<8, 2, false, true>; slot = 19; break;
      case 4 * 2: kern = fused_row_kernel<8, 4, false, true>; slot = 20; break;
      case 8 * 2: kern = fused_row_kernel<8, 8, false, true>; slot = 21; break;
      case 1 * 2 + 1: kern = fused_row_kernel<8, 1, true, true>; slot = 22; break;
      case 2 * 2 + 1: kern = fused_row_kernel<8, 2, true, true>; slot = 23; break;
      default: return hipErrorInvalidValue;
    }
  } else switch ((s.k_group * 4 + s.bits) * 2 + (vch ? 1 : 0)) {
    case (32 * 4 + 1) * 2: kern = fused_row_kernel<2, 1, false>; slot = 0; break;
    case (64 * 4 + 1) * 2: kern = fused_row_kernel<4, 1, false>; slot = 1; break;
    case (128 * 4 + 1) * 2: kern = fused_row_kernel<8, 1, false>; slot = 2; break;
    case (32 * 4 + 2) * 2: kern = fused_row_kernel<2, 2, false>; slot = 3; break;
    case (64 * 4 + 2) * 2: kern = fused_row_kernel<4, 2, false>; slot = 4; break;
    case (128 * 4 + 2) * 2: kern = fused_row_kernel<8, 2, false>; slot = 5; break;
    case (32 * 4 + 1) * 2 + 1: kern = fused_row_kernel<2, 1, true>; slot = 6; break;
    case (64 * 4 + 1) * 2 + 1: kern = fused_row_kernel<4, 1, true>; slot = 7; break;
    case (128 * 4 + 1) * 2 + 1: kern = fused_row_kernel<8, 1, true>; slot = 8; break;
    case (32 * 4 + 2) * 2 + 1: kern = fused_row_kernel<2, 2, true>; slot = 9; break;
    case (64 * 4 + 2) * 2 + 1: kern = fused_row_kernel<4, 2, true>; slot = 10; break;
    case (128 * 4 + 2) * 2 + 1: kern = fused_row_kernel<8, 2, true>; slot = 11; break;
    case (32 * 4 + 4) * 2: kern = fused_row_kernel<2, 4, false>; slot = 12; break;
    case (64 * 4 + 4) * 2: kern = fused_row_kernel<4, 4, false>; slot = 13; break;
    case (128 * 4 + 4) * 2: kern = fused_row_kernel<8, 4, false>; slot = 14; break;
    case (32 * 4 + 8) * 2: kern = fused_row_kernel<2, 8, false>; slot = 15; break;
    case (64 * 4 + 8) * 2: kern = fused_row_kernel<4, 8, false>; slot = 16; break;
    case (128 * 4 + 8) * 2: kern = fused_row_kernel<8, 8, false>; slot = 17; break;
    default: return hipErrorInvalidValue;
  }
  // long whole rows: three key groups in flight per wave
  if (plan.n_chunks == 1 && plan.nhb == 1 && !k_whole && !vch && s.k_group == 128 && s.bits <= 2 &&
      s.n_vis >= 48 * 128) {
    if (s.bits == 1) { kern = fused_row_kernel<8, 1, false, false, true, 3>; slot = 26; }
    else { kern = fused_row_kernel<8, 2, false, false, true, 3>; slot = 27; }
  }
  if (plan.n_chunks == 1 && plan.nhb == 1 && !k_whole && !vch && s.k_group == 32 && s.bits <= 2 &&
      s.n_vis >= 48 * 128) {
    if (s.bits == 1) { kern = fused_row_kernel<2, 1, false, false, true, 3>; slot = 28; }
    else { kern = fused_row_kernel<2, 2, false, false, true, 3>; slot = 29; }
  }
  // two head blocks per KV head: the twin workgroups share their lines through L2 (ordinary loads)
  if (plan.nhb > 1 && !k_whole && !vch && s.k_group == 128 && s.bits <= 2) {
    if (s.bits == 1) { kern = fused_row_kernel<8, 1, false, false, false>; slot = 24; }
    else { kern = fused_row_kernel<8, 2, false, false, false>; slot = 25; }
  }
  // the kernel's dynamic LDS limit is raised once per (device, kernel) and only ever grows;
  // concurrent callers may both raise it, which is harmless
  static std::atomic<size_t> configured[kMaxDevices][30];
  int dev = 0;
  hipError_t de = hipGetDevice(&dev);
  if (de != hipSuccess) return de;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (plan.lds > configured[dev][slot].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)plan.lds);
    if (e != hipSuccess) return e;
    size_t seen = configured[dev][slot].load(std::memory_order_relaxed);
    while (seen < plan.lds &&
           !configured[dev][slot].compare_exchange_weak(seen, plan.lds, std::memory_order_release)) {
    }
  }
  const size_t pieces = (size_t)s.B * s.Hkv * plan.n_chunks;
  const size_t blocks = plan.nhb > 1 ? (pieces + 7) / 8 * 8 * plan.nhb : pieces;
  if (blocks > 0x7fffffffu) return hipErrorInvalidConfiguration;
  a.n_pieces = (int)pieces;
  if (pieces * (size_t)plan.n_chunks >= ((size_t)1 << 32) || plan.nhb > 2) return hipErrorInvalidConfiguration;
  a.chunks_magic = plan.n_chunks == 1 ? 0u : (unsigned)((((unsigned long long)1 << 32) / (unsigned)plan.n_chunks) + 1);
  {
    const int n_units = s.n_vis / (s.k_group * a.unit), n_tblocks = (s.n_text + 63) / 64;
    a.units_base = n_units / plan.n_chunks;
    a.units_rem = n_units % plan.n_chunks;
    a.tblocks_base = n_tblocks / plan.n_chunks;
    a.tblocks_rem = n_tblocks % plan.n_chunks;
  }
  const dim3 grid((unsigned)blocks), block(kThreads);
  if (plan.n_chunks == 1 && plan.nhb == 1) {
    a.mode = kModeFull;
    kern<<<grid, block, plan.lds, stream>>>(a);
    return hipGetLastError();
  }
  if (calib.mode == CQ_CALIB_DYNAMIC) {
    a.mode = kModeExtrema;
    kern<<<grid, block, plan.lds, stream>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  a.mode = kModePartial;
  kern<<<grid, block, plan.lds, stream>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_combine(s.B * s.Hq, plan.n_chunks, kD, a.ws_partial, out, stream);
}

}  // namespace cq
