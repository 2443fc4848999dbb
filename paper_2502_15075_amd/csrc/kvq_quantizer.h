// The quantizer arithmetic shared by the bulk quantize-append kernel and the fused decode step.
//
// b-bit uniform scalar quantizer of App. B ("Preliminaries": scale factor, round, clip, reconstruct) of
// arXiv 2502.15075 in its group-wise asymmetric min-max form; the exact arithmetic is stated in kvq.h.
// Codes and scale/zero bytes must be identical wherever this is compiled, so floating-point contraction
// is switched off inside these functions whatever the translation unit's setting is, and every operation
// is a single IEEE binary32 operation (hipcc's default division is correctly rounded).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvq {

__device__ __forceinline__ float widen16(uint16_t bits, bool bf16) {
  if (bf16) return __uint_as_float((uint32_t)bits << 16);
  return (float)__builtin_bit_cast(_Float16, bits);
}

__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
  _Float16 h = (_Float16)f;  // v_cvt_f16_f32: round-to-nearest-even, subnormals kept
  return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

// ---- key rows ------------------------------------------------------------------------------------------------------------
// A key row takes 16 b bytes.  Widths 1, 2, 4, 8 (and 16-bit patterns): channel d at bits [d b, (d+1) b) of the row read
// as a little-endian bit string.  Widths 3 and 6 keep a power-of-two low part and the rest of every code in two runs:
// the row is cut into chunks of 32 channels (4 b bytes); with LO = 2 (b = 3) or 4 (b = 6) and HI = b - LO, channel x
// of a chunk has code mod 2^LO at bits [x LO, (x+1) LO) of the chunk and code >> LO at bits 32 LO + [x HI, (x+1) HI).
// (The attention kernel multiplies the two runs by the query separately: each is a field width it can unpack with
// one AND per two codes.)  Value codes of 3 and 6 bits are split the same way, one level up: a 32-token block is the
// block of the low parts followed by the block of the high parts.
template <int B> __host__ __device__ constexpr int code_lo_bits() { return B == 3 ? 2 : B == 6 ? 4 : B; }
template <int B> __host__ __device__ constexpr int code_hi_bits() { return B - code_lo_bits<B>(); }

// n-bit fields of the 8 codes, first code lowest: bits [shift, shift + N) of every code (MASK: the codes have bits
// above shift + N; otherwise nothing needs to be cut off)
template <int N, bool MASK> __device__ __forceinline__ uint32_t pack8(const uint32_t codes[8], int shift) {
  uint32_t w = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    uint32_t c = codes[e] >> shift;
    if (MASK) c &= (1u << N) - 1u;
    w |= c << (N * e);
  }
  return w;
}
// NT: a streaming store (the bulk append writes planes that nothing reads back soon; marked so, its stores and loads
// leave the caches to data that is reused, and the memory system takes the mixed read/write stream about a tenth faster)
template <int NBYTES, bool NT = false> __device__ __forceinline__ void store_bytes(uint8_t* p, uint32_t w) {
  if (NT) {
    if (NBYTES == 1) __builtin_nontemporal_store((uint8_t)w, p);
    else if (NBYTES == 2) __builtin_nontemporal_store((uint16_t)w, reinterpret_cast<uint16_t*>(p));
    else __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(p));
    return;
  }
  if (NBYTES == 1) *p = (uint8_t)w;
  else if (NBYTES == 2) *reinterpret_cast<uint16_t*>(p) = (uint16_t)w;
  else *reinterpret_cast<uint32_t*>(p) = w;
}
template <int NBYTES> __device__ __forceinline__ uint32_t load_bytes(const uint8_t* p) {
  if (NBYTES == 1) return *p;
  if (NBYTES == 2) return *reinterpret_cast<const uint16_t*>(p);
  return *reinterpret_cast<const uint32_t*>(p);
}

// Store the 8 codes of channels 8*lane16 .. 8*lane16+7 of one key row (rowp: first byte of the row).
template <int BK, bool NT = false>
__device__ __forceinline__ void store_key_codes(uint8_t* rowp, int lane16, const uint32_t codes[8]) {
  constexpr int LO = code_lo_bits<BK>(), HI = code_hi_bits<BK>();
  if constexpr (BK == 8) {
    const uint32_t w0 = codes[0] | (codes[1] << 8) | (codes[2] << 16) | (codes[3] << 24);
    const uint32_t w1 = codes[4] | (codes[5] << 8) | (codes[6] << 16) | (codes[7] << 24);
    if constexpr (NT) {
      typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
      u32x2 w; w.x = w0; w.y = w1;
      __builtin_nontemporal_store(w, reinterpret_cast<u32x2*>(rowp) + lane16);
    } else {
      reinterpret_cast<uint2*>(rowp)[lane16] = make_uint2(w0, w1);
    }
  } else if constexpr (HI == 0) {
    store_bytes<BK, NT>(rowp + lane16 * BK, pack8<BK, false>(codes, 0));          // 8 codes of b bits = b bytes
  } else {
    uint8_t* chunk = rowp + (lane16 >> 2) * (4 * BK);                      // 4 lanes = 32 channels = one chunk
    store_bytes<LO, NT>(chunk + (lane16 & 3) * LO, pack8<LO, true>(codes, 0));
    store_bytes<HI, NT>(chunk + 4 * LO + (lane16 & 3) * HI, pack8<HI, false>(codes, LO));
  }
}

// The 8 codes of channels 8*oct .. 8*oct+7 of a key row.
template <int B> __device__ __forceinline__ void load_key_codes(const uint8_t* rowp, int oct, uint32_t code[8]) {
  constexpr int LO = code_lo_bits<B>(), HI = code_hi_bits<B>();
  if constexpr (B == 16) {
    const uint4 w = *reinterpret_cast<const uint4*>(rowp + oct * 16);
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) code[e] = (ww[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
  } else if constexpr (B == 8) {
    const uint2 w = *reinterpret_cast<const uint2*>(rowp + oct * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) code[e] = ((e < 4 ? w.x : w.y) >> (8 * (e & 3))) & 0xFFu;
  } else if constexpr (HI == 0) {
    const uint32_t w = load_bytes<B>(rowp + oct * B);
#pragma unroll
    for (int e = 0; e < 8; ++e) code[e] = (w >> (B * e)) & ((1u << B) - 1u);
  } else {
    const uint8_t* chunk = rowp + (oct >> 2) * (4 * B);
    const uint32_t lo = load_bytes<LO>(chunk + (oct & 3) * LO), hi = load_bytes<HI>(chunk + 4 * LO + (oct & 3) * HI);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      code[e] = ((lo >> (LO * e)) & ((1u << LO) - 1u)) | (((hi >> (HI * e)) & ((1u << HI) - 1u)) << LO);
  }
}

// ---- randomized Hadamard rotation of a 128-channel row (Sec. 4 "Integration with Rotation-Based Methods") ----
// The row is held 8 consecutive channels per lane by 16 neighbouring lanes (lane16 = channel / 8).  R = H diag(s) /
// sqrt(128): signs, then the butterflies over strides 1, 2, 4 (inside the lane) and 8, 16, 32, 64 (partner lane
// lane16 ^ stride/8), each one binary32 add and one subtract (lower index minus higher index), then the scale.

constexpr float kRotScale = 0.08838834764831845f;   // binary32(1/sqrt(128))

// The 8 sign bits of the channels of lane16 (bit e set: channel 8*lane16 + e is negated).
__device__ __forceinline__ uint32_t rot_sign_bits(const uint32_t signs[4], int lane16) {
  const int w = lane16 >> 2;
  const uint32_t word = w == 0 ? signs[0] : w == 1 ? signs[1] : w == 2 ? signs[2] : signs[3];
  return (word >> (8 * (lane16 & 3))) & 0xFFu;
}

__device__ __forceinline__ void hadamard8x16(float x[8], int lane16) {
#pragma clang fp contract(off)
#pragma unroll
  for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if ((i & h) == 0) {
        const float a = x[i], b = x[i + h];
        x[i] = a + b;
        x[i + h] = a - b;
      }
  }
#pragma unroll
  for (int m = 1; m < 16; m <<= 1) {
    const bool upper = (lane16 & m) != 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float o = __shfl_xor(x[e], m, 16);
      x[e] = upper ? o - x[e] : x[e] + o;
    }
  }
}

// x <- R x
__device__ __forceinline__ void rotate8(float x[8], int lane16, uint32_t sign_bits) {
#pragma clang fp contract(off)
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = (sign_bits >> e) & 1u ? -x[e] : x[e];
  hadamard8x16(x, lane16);
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = x[e] * kRotScale;
}

// x <- R^T x
__device__ __forceinline__ void unrotate8(float x[8], int lane16, uint32_t sign_bits) {
#pragma clang fp contract(off)
  hadamard8x16(x, lane16);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float v = x[e] * kRotScale;
    x[e] = (sign_bits >> e) & 1u ? -v : v;
  }
}

// log2 of the lanes per group (4, 8 or 16 lanes of 8 channels: groups of 32, 64, 128 channels)
__device__ __forceinline__ int lpg_shift(int lanes_per_group) { return lanes_per_group == 4 ? 2 : lanes_per_group == 8 ? 3 : 4; }

// Minimum / maximum written as the machine instructions themselves (inputs are finite by contract, so the
// canonicalizing copies a C fmin / fmax needs are dead weight; -0 orders below +0 and is folded away afterwards).
__device__ __forceinline__ float min3f(float a, float b, float c) {
  float r; asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c)); return r;
}
__device__ __forceinline__ float max3f(float a, float b, float c) {
  float r; asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c)); return r;
}
__device__ __forceinline__ float min2f(float a, float b) { float r; asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
__device__ __forceinline__ float max2f(float a, float b) { float r; asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b)); return r; }
// Value of x in the lane a data-parallel-primitive control word selects (quad permutes and mirrors of a 16-lane
// row).  The builtin, not assembly: the compiler then keeps the wait states such an instruction needs.
template <int CTRL>
__device__ __forceinline__ float lane_dpp(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}

// ---- the two divisions of the quantizer, correctly rounded in three operations each ---------------------------------
// (mx - mn) / levels with levels = 2^b - 1 in {1, 3, 7, 15, 63, 255}: with c = RN(1 / levels), q0 = RN(x c),
// r = x - levels q0 (one fused multiply-add, exact), q1 = RN(q0 + r c) is the correctly rounded quotient (the classical
// correction step for a correctly rounded reciprocal; checked against IEEE division for every non-negative finite
// binary32 x and each of these divisors on a CPU).
__device__ __forceinline__ float inv_levels(int bits) {
  return bits == 4 ? 1.0f / 15.0f : bits == 2 ? 1.0f / 3.0f : bits == 8 ? 1.0f / 255.0f
       : bits == 3 ? 1.0f / 7.0f : bits == 6 ? 1.0f / 63.0f : 1.0f;          // (constants: rounded by the compiler)
}
__device__ __forceinline__ float div_levels(float x, float levels, float c) {
  const float q0 = x * c;
  const float r = __builtin_fmaf(-levels, q0, x);
  float q1 = __builtin_fmaf(r, c, q0);
  // The quotient is rounded to binary32 here and to binary16 afterwards.  Left to itself the compiler merges this
  // multiply-add with the conversion that follows into one mixed-precision instruction, which rounds the exact sum
  // once, straight to binary16, and lands on the other side of a tie: the value is made opaque so that it cannot.
  asm("" : "+v"(q1));
  return q1;
}
// 1 / s for a stored scale s (a positive binary16 value widened to binary32): one refinement of the hardware's
// reciprocal approximation, y1 = y0 + y0 (1 - s y0).  This is the correctly rounded reciprocal for every one of the
// 31743 possible scales on gfx950 (kvq_selftest_quantizer checks exactly that on the device it runs on); it is not for
// arbitrary binary32 inputs.
__device__ __forceinline__ float rcp_scale(float s) {
  const float y0 = __builtin_amdgcn_rcpf(s);
  const float e = __builtin_fmaf(-s, y0, 1.0f);
  return __builtin_fmaf(e, y0, y0);
}

// Quantize 8 consecutive elements held by this lane; the group spans `lanes_per_group`
// neighbouring lanes (a power of two <= 16, aligned).  Returns the 8 codes, and the stored
// scale/zero patterns through S, Z.
__device__ __forceinline__ void quantize8(const float x[8], int bits, int lanes_per_group, uint32_t codes[8],
                                          uint16_t* S, uint16_t* Z) {
#pragma clang fp contract(off)
  float mn = min3f(min3f(x[0], x[1], x[2]), min3f(x[3], x[4], x[5]), min2f(x[6], x[7]));
  float mx = max3f(max3f(x[0], x[1], x[2]), max3f(x[3], x[4], x[5]), max2f(x[6], x[7]));
  // the group's lanes are an aligned run of 4, 8 or 16 inside a 16-lane row: two quad exchanges, then the mirror
  // images of the 8- and 16-lane runs (after the quad steps every quad is uniform, so a mirror is as good as an xor)
  // Each step is one instruction per bound: the minimum (maximum) of a register and its own lane-permuted copy.  A
  // permuted read needs two wait states after the write of its source, which the compiler counts for its own
  // instructions only; here they are written out: a pause in front of each block (five states in front of the first,
  // which also covers an execution mask written by a vector compare just before; two in front of the others), and
  // inside the first block the other bound's instruction plus a one-state pause between a write and its permuted read.
  asm("s_nop 4\n\t"
      "v_min_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
      "s_nop 0\n\t"
      "v_min_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
      "v_max_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
      : "+v"(mn), "+v"(mx));
  if (lanes_per_group >= 8)
    asm("s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf"
        : "+v"(mn), "+v"(mx));
  if (lanes_per_group >= 16)
    asm("s_nop 1\n\t"
        "v_min_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
        "v_max_f32_dpp %1, %1, %1 row_mirror row_mask:0xf bank_mask:0xf"
        : "+v"(mn), "+v"(mx));
  if (mn == 0.0f) mn = 0.0f;  // -0 -> +0
  const float levels = (float)((1 << bits) - 1);
  float s32 = div_levels(mx - mn, levels, inv_levels(bits));
  uint16_t sb = f32_to_f16_bits(s32);
  if ((sb & 0x7FFFu) == 0) sb = 0;
  uint16_t zb = f32_to_f16_bits(mn);
  float s = widen16(sb, false), z = widen16(zb, false);
  *S = sb; *Z = zb;
  // a scale of 0 (constant group, or a range that underflows binary16): every code is 0, which a factor of 0 in place
  // of the reciprocal gives without a branch ((x - z) is finite, its product with 0 is +-0)
  float rcp = rcp_scale(s);
  if (s == 0.0f) rcp = 0.0f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float t = (x[e] - z) * rcp;
    float q = rintf(t);
    q = __builtin_amdgcn_fmed3f(q, 0.0f, levels);     // clip to [0, levels] in one instruction
    codes[e] = (uint32_t)q;
  }
}

// Value scales of 64 and more (a group range of 64 (2^b - 1) and up: legal, far from anything a model produces) need
// room in the attention kernel's binary16 weights.  Every kernel that stores a value scale raises the stream's entry of
// kvq_cache.v_scale_exp to the scale's exponent field when it is that large (a rare atomic; ordinary scales cost one
// comparison per group).  S: the stored binary16 pattern.
__device__ __forceinline__ void note_value_scale(int32_t* stream_exp, uint16_t S) {
  if (S >= 0x5400u) atomicMax(stream_exp, (int32_t)(S >> 10));      // 0x5400 = 64.0
}

// The same quantizer for a group that is not spread over neighbouring lanes (channel-wise key groups: the group runs
// over tokens): stored scale/zero patterns from the group's minimum and maximum, then one code at a time.
__device__ __forceinline__ void group_scale_zero(float mn, float mx, int bits, uint16_t* S, uint16_t* Z) {
#pragma clang fp contract(off)
  if (mn == 0.0f) mn = 0.0f;  // -0 -> +0
  const float levels = (float)((1 << bits) - 1);
  const float s32 = div_levels(mx - mn, levels, inv_levels(bits));
  uint16_t sb = f32_to_f16_bits(s32);
  if ((sb & 0x7FFFu) == 0) sb = 0;
  *S = sb;
  *Z = f32_to_f16_bits(mn);
}

// s, z: the stored scale/zero widened; rcp = 1 / s (unused when s == 0); levels = 2^bits - 1.
__device__ __forceinline__ uint32_t group_code(float x, float s, float z, float rcp, float levels) {
#pragma clang fp contract(off)
  if (s == 0.0f) return 0u;
  const float t = (x - z) * rcp;
  float q = rintf(t);
  q = fminf(fmaxf(q, 0.0f), levels);
  return (uint32_t)q;
}

}  // namespace kvq
